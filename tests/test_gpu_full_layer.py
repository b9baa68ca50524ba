"""GPU parity of the full-layer-parallel fuzzy step (the ablation of the paper's App. B) against
the CPU oracle in the same mode: chain steps and tree levels, logits, hidden states and every
stored k, v, then calibration on top.  Tolerances as in test_gpu_parity.py."""
import numpy as np
import pytest

import easyspec_synth as synth
from test_gpu_parity import TOL, IdCheck, kv_check

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device; none is visible")
    import gpu_harness
    return gpu_harness


def full_layer_parity(oracle, gpu, cfg, seed, bounds, prompt_len, n_steps, kv_prefix=0, batch=1):
    tol = TOL[cfg["dtype"]]
    w = synth.make_weights(cfg, seed)
    max_ctx = kv_prefix + prompt_len + 2 * n_steps + 40
    model = oracle.Model(cfg, w, max_ctx)
    so = [oracle.Sequence(model) for _ in range(batch)]
    g = gpu.GpuDrafter(cfg, w, max_batch=batch, max_ctx=max_ctx, max_calib=16)
    g.set_groups(bounds)
    g.set_full_layer(True)
    ids = IdCheck(cfg["dtype"])
    try:
        for b in range(batch):
            so[b].set_full_layer(True)
            if kv_prefix:
                k, v = synth.make_kv_prefix(cfg, seed + 9 + b, kv_prefix)
                so[b].import_kv(k, v)
                g.import_kv(b, k, v)
            prompt = synth.make_tokens(seed + 1 + b, prompt_len + 3 * b, cfg["vocab"])
            want = so[b].calibrate(prompt)                      # calibration is layer-sequential in both modes
            _, got = g.prefill(b, prompt)
            gpu.assert_close(got, want, tol)
        toks = synth.make_tokens(seed + 5, n_steps * batch, cfg["vocab"]).reshape(n_steps, batch)
        # what Alg. 2 would give for the first step: a different function when a set has several layers
        alg2 = so[0].clone()
        alg2.set_full_layer(False)
        other = alg2.fuzzy_step(bounds, toks[0, 0])
        for j in range(n_steps):
            gt, gl = g.draft_step({b: int(toks[j, b]) for b in range(batch)})
            if j == 0 and max(np.diff(bounds)) > 1:
                assert gpu.rel_l2(gl[0], other) > 20 * tol
            hid = g.hidden()
            for b in range(batch):
                wl, wh = so[b].fuzzy_step(bounds, toks[j, b], want_hidden=True)
                gpu.assert_close(gl[b], wl, tol, f"step {j} sequence {b} logits")
                gpu.assert_close(hid[b], wh, tol, "hidden state")
                ids(oracle, gt[b], wl)
        for b in range(batch):
            kv_check(gpu, g, so[b], b, so[b].precise + so[b].fuzzy, tol)
        # a tree level and a calibration on top, first sequence
        for b in range(batch):
            so[b].calibrate([3, 4])
        g.calibrate({b: [3, 4] for b in range(batch)})
        wl = so[0].fuzzy_tree_step(bounds, [5, 6, 7], [-1, -1, -1])
        _, gl = g.draft_tree_step({0: ([5, 6, 7], [-1, -1, -1])})
        gpu.assert_close(gl[0], wl, tol, "tree level")
        wl = so[0].fuzzy_tree_step(bounds, [8, 9], [0, 2])
        _, gl = g.draft_tree_step({0: ([8, 9], [0, 2])})
        gpu.assert_close(gl[0], wl, tol, "second tree level")
        kv_check(gpu, g, so[0], 0, so[0].precise + so[0].fuzzy, tol)
    finally:
        g.close()


@pytest.mark.parametrize("bounds", [[0, 1, 3, 4], [0, 4], [0, 2, 4], [0, 1, 2, 3, 4]])
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_full_layer_tiny(oracle, gpu, bounds, dtype):
    full_layer_parity(oracle, gpu, synth.model_shape("tiny", dtype=dtype), 600, bounds, 40, 3)


def test_full_layer_qwen_shape_batch2(oracle, gpu):
    full_layer_parity(oracle, gpu, synth.model_shape("tiny_qwen", dtype="bf16"), 610, [0, 1, 4, 5], 37, 3, batch=2)


def test_full_layer_8b_shape_reduced_depth(oracle, gpu):
    """8B layer shape, 6 layers as sets {0}, {1-4}, {5}; 2048-slot synthetic prefix."""
    cfg = synth.model_shape("llama3_8b", n_layers=6, vocab=4096)
    full_layer_parity(oracle, gpu, cfg, 620, [0, 1, 5, 6], 5, 2, kv_prefix=2048)


def test_mode_switch_and_bad_mode(gpu):
    import paper_2502_02493_amd as es
    cfg = synth.model_shape("tiny")
    g = gpu.GpuDrafter(cfg, synth.make_weights(cfg, 1), max_batch=1, max_ctx=64, max_calib=8)
    try:
        g.set_groups([0, 1, 3, 4])
        g.calibrate({0: [1, 2, 3]})
        _, a = g.draft_step({0: 5})
        es.easyspec_truncate(g.ctx, 0, 3)
        g.set_full_layer(True)
        _, b = g.draft_step({0: 5})
        es.easyspec_truncate(g.ctx, 0, 3)
        g.set_full_layer(False)
        _, a2 = g.draft_step({0: 5})
        assert np.array_equal(a, a2) and not np.array_equal(a, b)
        with pytest.raises(es.EasySpecError) as e:
            es.easyspec_set_parallel_mode(g.ctx, 2)
        assert e.value.code == es.EASYSPEC_EINVAL
    finally:
        g.close()
