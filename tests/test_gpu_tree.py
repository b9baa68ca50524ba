"""GPU parity of the token-tree draft step (paper Sec. 3.1 last paragraph, App. C) against the
CPU oracle: logits, hidden states and every stored k, v of every node, level by level, on the
same seeded weights, tokens and tree shapes; then calibration on top of the tree.  Tolerances as
in test_gpu_parity.py."""
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


def make_tree(seed, widths, vocab):
    """Levels of the given widths; every node's parent is drawn among the nodes of the level above
    (-1 on the first level), so that some nodes have several children and some none."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 99]))
    levels, first = [], 0
    for li, w in enumerate(widths):
        if li == 0:
            parents = [-1] * w
        else:
            prev = list(range(first - widths[li - 1], first))
            parents = sorted(int(rng.choice(prev)) for _ in range(w))
        toks = [int(t) for t in rng.integers(0, vocab, w)]
        levels.append((toks, parents))
        first += w
    return levels


def tree_parity(oracle, gpu, cfg, seed, bounds, prompt_len, widths, max_ctx=None, kv_prefix=0, make_levels=make_tree):
    tol = TOL[cfg["dtype"]]
    w = synth.make_weights(cfg, seed)
    total = sum(widths)
    max_ctx = max_ctx or (kv_prefix + prompt_len + total + 24)
    so = oracle.Sequence(oracle.Model(cfg, w, max_ctx))
    g = gpu.GpuDrafter(cfg, w, max_batch=1, max_ctx=max_ctx, max_calib=16)
    g.set_groups(bounds)
    ids = IdCheck(cfg["dtype"])
    try:
        if kv_prefix:
            k, v = synth.make_kv_prefix(cfg, seed + 9, kv_prefix)
            so.import_kv(k, v)
            g.import_kv(0, k, v)
        prompt = synth.make_tokens(seed + 1, prompt_len, cfg["vocab"])
        so.calibrate(prompt)
        g.prefill(0, prompt)
        P = so.precise
        for it in range(2):
            levels = make_levels(seed + 10 * it, widths, cfg["vocab"])
            for toks, parents in levels:
                wl, wh = so.fuzzy_tree_step(bounds, toks, parents, want_hidden=True)
                gt, gl = g.draft_tree_step({0: (toks, parents)})
                assert gl[0].shape == wl.shape
                gpu.assert_close(gl[0], wl, tol, "tree logits")
                for j in range(len(toks)):
                    gpu.assert_close(gl[0][j], wl[j], 4 * tol, f"tree logits node {j}")
                    ids(oracle, gt[0][j], wl[j])
                gpu.assert_close(g.hidden(), wh, tol, "tree hidden states")
            p, f = g.lens()
            assert (p[0], f[0]) == (so.precise, so.fuzzy) == (P, total)
            kv_check(gpu, g, so, 0, P + total, tol)                       # every node's k, v included
            calib = [int(t) for t in synth.make_tokens(seed + 20 + it, 3, cfg["vocab"])]
            wl = so.calibrate(calib)
            gt, gl = g.calibrate({0: calib})
            gpu.assert_close(gl[0], wl, tol, "calibration after a tree")
            P = so.precise
            kv_check(gpu, g, so, 0, P, tol)
        assert ids.checked >= total and ids.skipped <= max(2, ids.checked // 4), (ids.checked, ids.skipped)
    finally:
        g.close()


@pytest.mark.parametrize("bounds", [[0, 1, 3, 4], [0, 4]])
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_tree_tiny(oracle, gpu, bounds, dtype):
    tree_parity(oracle, gpu, synth.model_shape("tiny", dtype=dtype), 500, bounds, 70, [4, 4, 4, 4])


def test_tree_widths_of_the_ablation(oracle, gpu):
    """Tree widths 1, 4, 8, 12 (the paper's ablation, Sec. 4.3), five levels: up to 60 nodes."""
    cfg = synth.model_shape("tiny", dtype="bf16")
    for width in (1, 4, 8, 12):
        tree_parity(oracle, gpu, cfg, 510 + width, [0, 1, 3, 4], 33, [width] * 5)


def test_tree_qwen_shape_ragged(oracle, gpu):
    """7 query heads per KV head, bias, head_dim 64; a tree region that straddles an attention chunk boundary."""
    cfg = synth.model_shape("tiny_qwen", dtype="bf16")
    tree_parity(oracle, gpu, cfg, 520, [0, 1, 4, 5], 250, [3, 5, 2, 7])


def test_tree_8b_shape_reduced_depth_long_context(oracle, gpu):
    """8B layer shape at 3 layers, 2048-slot synthetic prefix (split-KV attention with a merge), width 8."""
    cfg = synth.model_shape("llama3_8b", n_layers=3, vocab=4096)
    tree_parity(oracle, gpu, cfg, 530, [0, 1, 3], 5, [8, 8, 8], kv_prefix=2048)


def test_tree_chunk_without_visible_slot(oracle, gpu, monkeypatch):
    """Fresh roots added after two levels see none of the earlier nodes: with the tree region starting on
    a batch boundary and one batch per split-KV chunk, the chunk that holds the first 32 nodes has no
    visible slot for them (a partial with maximum -inf that the merge must weigh with 0)."""
    monkeypatch.setenv("EASYSPEC_ATTN_MFMA", "0")
    monkeypatch.setenv("EASYSPEC_ATTN_NCH", "64")

    def levels_with_late_roots(seed, widths, vocab):
        levels = make_tree(seed, widths, vocab)
        toks, _ = levels[2]
        levels[2] = (toks, [-1] * len(toks))
        return levels

    for dtype, prompt_len in (("fp32", 288), ("bf16", 320)):      # 32 / 64 slots per batch at head_dim 64
        cfg = synth.model_shape("tiny", dtype=dtype)
        tree_parity(oracle, gpu, cfg, 540, [0, 1, 3, 4], prompt_len, [16, 16, 16, 16], make_levels=levels_with_late_roots)


def test_tree_two_sequences_ragged(oracle, gpu):
    """Two sequences with different contexts grow different trees in the same calls (3 + 2 nodes,
    then 4 + 5 nodes); a third call extends only the second sequence."""
    cfg = synth.model_shape("tiny", dtype="bf16")
    bounds = [0, 1, 3, 4]
    tol = TOL["bf16"]
    w = synth.make_weights(cfg, 540)
    model = oracle.Model(cfg, w, 160)
    so = [oracle.Sequence(model), oracle.Sequence(model)]
    g = gpu.GpuDrafter(cfg, w, max_batch=2, max_ctx=160, max_calib=16)
    g.set_groups(bounds)
    try:
        for b, n in ((0, 11), (1, 70)):
            prompt = synth.make_tokens(541 + b, n, cfg["vocab"])
            so[b].calibrate(prompt)
            g.prefill(b, prompt)
        calls = [{0: ([5, 6, 7], [-1, -1, -1]), 1: ([8, 9], [-1, -1])},
                 {0: ([1, 2, 3, 4], [0, 0, 2, 2]), 1: ([11, 12, 13, 14, 15], [0, 1, 1, 1, 0])},
                 {1: ([21, 22, 23], [2, 6, 6])}]
        for call in calls:
            gt, gl = g.draft_tree_step(call)
            for b, (toks, parents) in call.items():
                wl = so[b].fuzzy_tree_step(bounds, toks, parents)
                gpu.assert_close(gl[b], wl, tol, f"sequence {b}")
        p, f = g.lens()
        for b in (0, 1):
            assert (p[b], f[b]) == (so[b].precise, so[b].fuzzy)
            kv_check(gpu, g, so[b], b, so[b].precise + so[b].fuzzy, tol)
    finally:
        g.close()


def test_tree_error_paths(gpu):
    import paper_2502_02493_amd as es
    cfg = synth.model_shape("tiny")
    g = gpu.GpuDrafter(cfg, synth.make_weights(cfg, 1), max_batch=2, max_ctx=128, max_calib=8)
    try:
        def code(fn):
            with pytest.raises(es.EasySpecError) as e:
                fn()
            return e.value.code
        assert code(lambda: g.draft_tree_step({0: ([1], [-1])})) == es.EASYSPEC_ESTATE          # no context yet
        g.calibrate({0: [1, 2, 3], 1: [4, 5]})
        assert code(lambda: g.draft_tree_step({0: ([1], [0])})) == es.EASYSPEC_EINVAL           # parent does not exist
        g.draft_tree_step({0: ([1, 2], [-1, -1])})
        assert code(lambda: g.draft_tree_step({0: ([1, 2], [0, 2])})) == es.EASYSPEC_EINVAL     # parent in the same level
        assert code(lambda: g.draft_step({0: 1, 1: 2})) == es.EASYSPEC_ESTATE                   # chain step into a tree
        g.calibrate({0: [7]})
        g.draft_step({0: 1, 1: 2})
        assert code(lambda: g.draft_tree_step({1: ([1], [-1])})) == es.EASYSPEC_ESTATE          # tree after chain slots
        g.calibrate({0: [7], 1: [8]})
        assert code(lambda: g.draft_tree_step({0: (list(range(9)), [-1] * 9), 1: (list(range(9)), [-1] * 9)})) == es.EASYSPEC_ECAPACITY
        for lvl in range(4):
            g.draft_tree_step({0: (list(range(16)), [-1] * 16 if lvl == 0 else [0] * 16)})
        assert code(lambda: g.draft_tree_step({0: ([1], [0])})) == es.EASYSPEC_ECAPACITY        # 65th node
        p, f = g.lens()
        assert f[0] == 64
    finally:
        g.close()
