"""GPU parity with the matrix-core attention kernel forced on (it is otherwise chosen only for
launches with several columns of a sequence and enough work, which the small shapes of the other
test modules rarely reach): the same oracle comparisons as test_gpu_parity / test_gpu_tree /
test_gpu_full_layer, on bf16 models (the kernel serves bf16 caches only), head_dim 128 and 64,
1 / 2 / 7 query heads per KV head, ragged contexts, tree masks, batch 2."""
import os

import pytest

import easyspec_synth as synth
from test_gpu_parity import iteration_parity
from test_gpu_tree import tree_parity
from test_gpu_tree import test_tree_two_sequences_ragged as _two_sequences_ragged
from test_gpu_full_layer import full_layer_parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device; none is visible")
    import gpu_harness
    return gpu_harness


@pytest.fixture(autouse=True)
def force_mfma_attention():
    old = os.environ.get("EASYSPEC_ATTN_MFMA")
    os.environ["EASYSPEC_ATTN_MFMA"] = "2"
    yield
    if old is None:
        del os.environ["EASYSPEC_ATTN_MFMA"]
    else:
        os.environ["EASYSPEC_ATTN_MFMA"] = old


@pytest.mark.parametrize("bounds", [[0, 1, 3, 4], [0, 4]])
def test_iteration_tiny_bf16(oracle, gpu, bounds):
    """head_dim 64, 2 query heads per KV head; prompt 70 (two 64-slot super tiles, ragged), chunked prefill."""
    iteration_parity(oracle, gpu, synth.model_shape("tiny", dtype="bf16"), 700, bounds, 70, 4)


def test_iteration_qwen_shape(oracle, gpu):
    """7 query heads per KV head: two columns per MFMA tile (14 of 16 rows), QKV bias."""
    iteration_parity(oracle, gpu, synth.model_shape("tiny_qwen", dtype="bf16"), 710, [0, 1, 4, 5], 37, 5)


def test_iteration_head_dim_128_one_head_per_kv(oracle, gpu):
    cfg = synth.model_shape("tiny", dtype="bf16", head_dim=128, n_q_heads=2, n_kv_heads=2)
    iteration_parity(oracle, gpu, cfg, 720, [0, 1, 3, 4], 67, 3)
    iteration_parity(oracle, gpu, cfg, 721, [0, 1, 3, 4], 1, 3)


def test_long_prompt_several_sub_chunks(oracle, gpu):
    """Context beyond the single-chunk limit: split-KV partials of the MFMA kernel merged by the merge kernel."""
    cfg = synth.model_shape("tiny", dtype="bf16")
    iteration_parity(oracle, gpu, cfg, 730, [0, 1, 3, 4], 300, 4, n_iters=1)


@pytest.mark.parametrize("widths", [[4, 4, 4, 4], [12, 12, 12], [3, 5, 2, 7]])
def test_tree(oracle, gpu, widths):
    tree_parity(oracle, gpu, synth.model_shape("tiny", dtype="bf16"), 740 + len(widths), [0, 1, 3, 4], 70, widths)


def test_tree_qwen_shape_straddling_chunks(oracle, gpu):
    tree_parity(oracle, gpu, synth.model_shape("tiny_qwen", dtype="bf16"), 750, [0, 1, 4, 5], 250, [3, 5, 2, 7])


def test_tree_8b_shape_long_context(oracle, gpu):
    cfg = synth.model_shape("llama3_8b", n_layers=3, vocab=4096)
    tree_parity(oracle, gpu, cfg, 760, [0, 1, 3], 5, [8, 8, 8], kv_prefix=2048)


def test_full_layer_batch2(oracle, gpu):
    full_layer_parity(oracle, gpu, synth.model_shape("tiny_qwen", dtype="bf16"), 770, [0, 1, 4, 5], 37, 3, batch=2)


def test_tree_two_sequences_ragged(oracle, gpu):
    """Several groups per launch: two sequences of different length growing different trees."""
    _two_sequences_ragged(oracle, gpu)


def test_calibration_of_two_sequences_in_one_call(oracle, gpu):
    """Causal columns of two sequences in one pass (5 + 9 tokens: groups of 8, 1 and 5 columns at
    2 query heads per KV head), after fuzzy steps that must leave no trace."""
    from test_gpu_parity import TOL
    cfg = synth.model_shape("tiny", dtype="bf16")
    w = synth.make_weights(cfg, 780)
    model = oracle.Model(cfg, w, 200)
    so = [oracle.Sequence(model), oracle.Sequence(model)]
    g = gpu.GpuDrafter(cfg, w, max_batch=2, max_ctx=200, max_calib=16)
    g.set_groups([0, 1, 3, 4])
    try:
        for b, n in ((0, 90), (1, 131)):
            prompt = synth.make_tokens(781 + b, n, cfg["vocab"])
            so[b].calibrate(prompt)
            g.prefill(b, prompt)
        for t in (3, 4):
            g.draft_step({0: t, 1: t + 10})
            so[0].fuzzy_step([0, 1, 3, 4], t)
            so[1].fuzzy_step([0, 1, 3, 4], t + 10)
        toks = {0: [1, 2, 3, 4, 5], 1: [6, 7, 8, 9, 10, 11, 12, 13, 14]}
        _, gl = g.calibrate(toks)
        for b in (0, 1):
            gpu.assert_close(gl[b], so[b].calibrate(toks[b]), TOL["bf16"], f"sequence {b}")
    finally:
        g.close()
