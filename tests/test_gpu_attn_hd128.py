"""GPU parity of the vector attention kernel where its scores come from the matrix cores: bf16 caches,
head_dim 128, four, seven and eight query heads per KV head (probabilities passed on by quad broadcasts
with four heads, through the wave's LDS with more), with the matrix-core attention kernel switched off so
that calibrations and tree levels take this kernel too.  Small models of those head shapes, the same
oracle comparisons as test_gpu_parity / test_gpu_tree; the cases pick contexts that end in one chunk of
eight waves, in several chunks of full batches followed by short steps, and (a forced cut into two
chunks) in runs of several full batches per wave, where the next batch is requested ahead."""
import os

import pytest

import easyspec_synth as synth
from test_gpu_parity import iteration_parity
from test_gpu_tree import tree_parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device; none is visible")
    import gpu_harness
    return gpu_harness


@pytest.fixture(autouse=True)
def vector_attention_only(monkeypatch):
    monkeypatch.setenv("EASYSPEC_ATTN_MFMA", "0")
    yield


def head_shape(G, n_kv=1, **kw):
    """A 4-layer bf16 decoder with head_dim 128 and G query heads for each of n_kv KV heads."""
    return synth.model_shape("tiny", dtype="bf16", head_dim=128, n_q_heads=G * n_kv, n_kv_heads=n_kv,
                             d_model=128 * G * n_kv, d_ffn=1024, qkv_bias=int(G == 7), **kw)


@pytest.mark.parametrize("G, n_kv", [(4, 2), (7, 1), (8, 1)])
@pytest.mark.parametrize("prompt_len", [5, 37, 250, 300, 707])
def test_iteration(oracle, gpu, G, n_kv, prompt_len):
    """One context per launch shape: 5 and 37 slots (one short step; one chunk, eight waves), 250 (the
    longest single chunk), 300 and 707 (several chunks of four waves: full batches, then short steps)."""
    iteration_parity(oracle, gpu, head_shape(G, n_kv), 900 + G + prompt_len, [0, 1, 3, 4], prompt_len, 4,
                     n_iters=1 if prompt_len > 256 else 2)


@pytest.mark.parametrize("G, n_kv", [(4, 2), (7, 1)])
def test_runs_of_several_full_batches(oracle, gpu, monkeypatch, G, n_kv):
    """A context of 1500 slots cut into two chunks only: every wave walks five or six full batches, so the
    loop that requests the next batch while it works on the current one goes round several times."""
    monkeypatch.setenv("EASYSPEC_ATTN_NCH", "2")
    iteration_parity(oracle, gpu, head_shape(G, n_kv), 930 + G, [0, 2, 4], 1500, 3, n_iters=1)


@pytest.mark.parametrize("G, n_kv", [(4, 1), (7, 1), (8, 1)])
def test_tree(oracle, gpu, G, n_kv):
    """The kernel's tree-mask instantiation: levels of several widths over a prompt that straddles chunks."""
    tree_parity(oracle, gpu, head_shape(G, n_kv), 950 + G, [0, 1, 3, 4], 270, [3, 5, 2, 7])
    tree_parity(oracle, gpu, head_shape(G, n_kv), 960 + G, [0, 4], 40, [4, 4, 4])
