"""GPU parity at the benchmark shapes and in the batched / ragged / degenerate cases.

Full-depth 8B-shape runs are sampled (one iteration); the layer shapes of both model
families are also run at reduced depth so that the oracle can follow every step, with a
seeded synthetic KV prefix (imported by both sides) standing in for a long prefilled context.
"""
import numpy as np
import pytest

import easyspec_synth as synth

from tolerances import MARGIN, TOL

pytestmark = pytest.mark.gpu



@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device; none is visible")
    import gpu_harness
    return gpu_harness


def check_ids(oracle, dtype, got, want_logits, stats):
    want, margin = oracle.argmax(want_logits, with_margin=True)
    if stats is not None and margin > MARGIN[dtype] * float(np.std(want_logits)):
        assert int(got) == want
        stats[0] += 1
    elif stats is not None:
        stats[1] += 1
    return want


def groups(es, cfg, N, policy="aligned"):
    pol = es.EASYSPEC_POLICY_ALIGNED if policy == "aligned" else es.EASYSPEC_POLICY_PACKED
    return es.easyspec_default_groups(cfg["n_layers"], N, pol)


def one_iteration(oracle, gpu, cfg, seed, bounds, ctx_len, gamma, accept, max_ctx=None, plain=False):
    """Synthetic KV prefix of ctx_len slots, calibration of 2 tokens, gamma-1 fuzzy steps,
    calibration of `accept` drafted tokens + bonus.  Compares logits, hidden states, ids, KV.
    plain: against the oracle with unrounded activations (bf16 weights and cache only) at the
    tolerance required of a bf16 model; ids are then not compared (the sides decide in different precisions)."""
    import paper_2502_02493_amd  # noqa: F401
    tol, dt = (gpu.PLAIN_TOL if plain else TOL[cfg["dtype"]]), cfg["dtype"]
    w = synth.make_weights(cfg, seed)
    max_ctx = max_ctx or ctx_len + gamma + 16
    model = oracle.Model(cfg, w, max_ctx)
    if plain:
        model.set_rounding(oracle.ACT_PLAIN, dt == "bf16")
    so = oracle.Sequence(model)
    g = gpu.GpuDrafter(cfg, w, max_batch=1, max_ctx=max_ctx, max_calib=16)
    stats = None if plain else [0, 0]
    try:
        g.set_groups(bounds)
        k, v = synth.make_kv_prefix(cfg, seed + 1, ctx_len)
        so.import_kv(k, v)
        g.import_kv(0, k, v)
        toks = synth.make_tokens(seed + 2, 3, cfg["vocab"])
        wl = so.calibrate(toks[:2], all_rows=True)
        gt, gl = g.calibrate({0: list(toks[:2])}, all_rows=True)
        gpu.assert_close(gl[0], wl, tol, "calibration logits")
        drafted = [check_ids(oracle, dt, gt[0], wl[-1], stats)]
        for _ in range(gamma - 1):
            wl, wh = so.fuzzy_step(bounds, drafted[-1], want_hidden=True)
            gtok, glog = g.draft_step({0: drafted[-1]})
            gpu.assert_close(glog[0], wl, tol, "fuzzy logits")
            gpu.assert_close(g.hidden()[0], wh, tol, "fuzzy hidden state")
            drafted.append(check_ids(oracle, dt, gtok[0], wl, stats))
        n = so.precise + so.fuzzy
        gk, gv = g.export_kv(0, n)
        # only the slots written by this run; the imported prefix is trivially equal
        assert gpu.rel_l2(gk[:, :, ctx_len:], so.K[:, :, ctx_len:n]) < max(tol, 4e-3 if dt == "bf16" else 0), "K"
        assert gpu.rel_l2(gv[:, :, ctx_len:], so.V[:, :, ctx_len:n]) < max(tol, 4e-3 if dt == "bf16" else 0), "V"
        calib = drafted[:accept] + [int(toks[2])]
        wl, wh = so.calibrate(calib, all_rows=True, want_hidden=True)
        gt, gl = g.calibrate({0: calib}, all_rows=True)
        gpu.assert_close(gl[0], wl, tol, "bonus calibration logits")
        gpu.assert_close(g.hidden(), wh, tol, "bonus calibration hidden")
        check_ids(oracle, dt, gt[0], wl[-1], stats)
        p, f = g.lens()
        assert (int(p[0]), int(f[0])) == (so.precise, 0) == (ctx_len + 2 + accept + 1, 0)
        assert plain or stats[0] >= 1
    finally:
        g.close()
    return stats


def test_llama3_8b_layer_shape_reduced_depth(oracle, gpu):
    """8B layer shape, 6 layers, sets {0},{1,2,3},{4},{5} (aligned, N=4), context 256, gamma 5."""
    import paper_2502_02493_amd as es
    cfg = synth.model_shape("llama3_8b", n_layers=6, vocab=8192)
    b = groups(es, cfg, 4)
    assert list(b) == [0, 1, 4, 5, 6]
    one_iteration(oracle, gpu, cfg, 500, b, 256, 5, accept=3)


def test_llama3_8b_layer_shape_reduced_depth_against_plain_oracle(oracle, gpu):
    """The same case against the oracle that knows nothing of two-term activations or of the norm carried
    in two parts: rel-L2 <= 2e-2, the required bar."""
    import paper_2502_02493_amd as es
    cfg = synth.model_shape("llama3_8b", n_layers=6, vocab=8192)
    one_iteration(oracle, gpu, cfg, 500, groups(es, cfg, 4), 256, 5, accept=3, plain=True)


@pytest.mark.parametrize("rows", [13, 15])
@pytest.mark.parametrize("dtype,accept", [("fp32", 2), ("bf16", 2), ("bf16", 10)])
def test_gate_up_weight_tiles_of_fewer_rows(oracle, gpu, monkeypatch, rows, dtype, accept):
    """The gate and up matrices packed in tiles of 13 / 15 rows instead of 16 (what the library picks
    by itself when that evens out the workgroups per CU: 14 rows at the 8B width, 15 at Qwen2-7B's):
    1024 rows leave a ragged last tile either way.  The 11-token calibration of the last case takes
    the two-fragment kernel, whose workgroups hold two row tiles of each matrix: 79 and 69 tiles leave
    the last workgroup with one."""
    monkeypatch.setenv("EASYSPEC_TILE_ROWS", str(rows))
    monkeypatch.setenv("EASYSPEC_PAIR_TILES", "1")  # the library pairs only launches that fill the CUs
    cfg = synth.model_shape("tiny", dtype=dtype)
    one_iteration(oracle, gpu, cfg, 560 + rows, [0, 1, 3, 4], 40, accept + 2, accept=accept)


@pytest.mark.parametrize("shape", ["tiny", "tiny_qwen"])
@pytest.mark.parametrize("pair", [0, 1])
def test_two_fragment_passes_with_and_without_paired_tiles(oracle, gpu, monkeypatch, shape, pair):
    """Passes of more than 8 columns (a 12-token calibration, bf16): every weight kernel with one row
    tile per workgroup and with two (what the library takes where the halved launch still fills the
    CUs: QKV and O of stacked sets, gate/up, LM head)."""
    monkeypatch.setenv("EASYSPEC_PAIR_TILES", str(pair))
    cfg = synth.model_shape(shape, dtype="bf16")
    one_iteration(oracle, gpu, cfg, 590 + pair, [0, 1, 3, cfg["n_layers"]], 70, 13, accept=11)


@pytest.mark.parametrize("rows", [8, 12, 16])
@pytest.mark.parametrize("shape", ["tiny", "tiny_qwen"])
def test_qkv_weight_tiles_of_fewer_rotation_pairs(oracle, gpu, monkeypatch, rows, shape):
    """The QKV matrices packed in tiles of 8 / 12 / 16 rotation pairs (12 is what the library picks
    at the 8B and Qwen2-7B widths, 16 for small models), bf16, with and without QKV bias; tiles of 12
    straddle head boundaries and leave a ragged last tile."""
    monkeypatch.setenv("EASYSPEC_QKV_TILE_ROWS", str(rows))
    cfg = synth.model_shape(shape, dtype="bf16")
    one_iteration(oracle, gpu, cfg, 580 + rows, [0, 1, 3, cfg["n_layers"]], 40, 4, accept=2)


@pytest.mark.parametrize("N,n_layers", [(2, 9), (4, 9), (7, 16), (8, 18)])
def test_qwen2_7b_layer_shape_reduced_depth(oracle, gpu, N, n_layers):
    """Qwen2-7B layer shape (7 query heads per KV head, QKV bias), group sizes 2/4/7 and the library's
    largest (8) at a depth where the aligned rule really yields a set of that many layers (16 layers,
    N=7: 0 | 1-6 | 7-13 | 14 | 15; 18 layers, N=8: 0 | 1-7 | 8-15 | 16 | 17), vocabulary not a multiple
    of 16, context 300 (ragged against every tile size)."""
    import paper_2502_02493_amd as es
    cfg = synth.model_shape("qwen2_7b", n_layers=n_layers, vocab=5003)
    b = groups(es, cfg, N)
    assert int(np.max(np.diff(b))) == N, list(b)
    one_iteration(oracle, gpu, cfg, 510 + N, b, 300, 5, accept=5 if N >= 7 else 1)


@pytest.mark.parametrize("ctx_len", [4096, 8191])
def test_calibration_lengths_long_context(oracle, gpu, ctx_len):
    """Calibration-dominant case at reduced depth: every calibration length 1..9 (gamma 8) behind
    a long synthetic context, partial KV rewrites included (what is accepted varies per round)."""
    import paper_2502_02493_amd as es
    cfg = synth.model_shape("llama3_8b", n_layers=2, vocab=4096)
    w = synth.make_weights(cfg, 520)
    max_ctx = ctx_len + 80
    so = oracle.Sequence(oracle.Model(cfg, w, max_ctx))
    g = gpu.GpuDrafter(cfg, w, max_batch=1, max_ctx=max_ctx, max_calib=9)
    try:
        bounds = groups(es, cfg, 4)
        g.set_groups(bounds)
        k, v = synth.make_kv_prefix(cfg, 521, ctx_len)
        so.import_kv(k, v); g.import_kv(0, k, v)
        toks = synth.make_tokens(522, 64, cfg["vocab"])
        at = 0
        for m in (9, 1, 5, 2, 8, 3, 7, 4, 6):
            for j in range(2):                         # fuzzy slots that the calibration must drop
                so.fuzzy_step(bounds, int(toks[at])); g.draft_step({0: int(toks[at])}); at += 1
            calib = [int(t) for t in toks[at: at + m]]
            wl = so.calibrate(calib, all_rows=True)
            gt, gl = g.calibrate({0: calib}, all_rows=True)
            gpu.assert_close(gl[0], wl, TOL["bf16"], f"calibration of {m} tokens")
            p, f = g.lens()
            assert (int(p[0]), int(f[0])) == (so.precise, 0)
        n = so.precise
        gk, gv = g.export_kv(0, n)
        assert gpu.rel_l2(gk[:, :, ctx_len:], so.K[:, :, ctx_len:n]) < 4e-3
        assert gpu.rel_l2(gv[:, :, ctx_len:], so.V[:, :, ctx_len:n]) < 4e-3
    finally:
        g.close()


def test_batch4_ragged_long_contexts(oracle, gpu):
    """Long-context batched draft at reduced depth: 4 sequences with contexts
    4096/8192/16384/32768 (ragged: minus 0/1/17/63), group size 4, fuzzy steps for all four at
    once, then a calibration that skips one sequence."""
    import paper_2502_02493_amd as es
    cfg = synth.model_shape("llama3_8b", n_layers=3, vocab=4096)
    w = synth.make_weights(cfg, 530)
    ctxs = [4096, 8191, 16367, 32705]
    max_ctx = 32768
    model = oracle.Model(cfg, w, max_ctx)
    seqs = [oracle.Sequence(model) for _ in ctxs]
    g = gpu.GpuDrafter(cfg, w, max_batch=4, max_ctx=max_ctx, max_calib=6)
    try:
        bounds = np.array([0, 3], np.int32)            # one 3-layer set: the grouped-attention case
        g.set_groups(bounds)
        for b, n in enumerate(ctxs):
            k, v = synth.make_kv_prefix(cfg, 531, n, seq=b)
            seqs[b].import_kv(k, v); g.import_kv(b, k, v)
        toks = synth.make_tokens(532, 64, cfg["vocab"]).reshape(4, 16)
        for step in range(3):
            feed = {b: int(toks[b, step]) for b in range(4)}
            gt, gl = g.draft_step(feed)
            for b in range(4):
                wl = seqs[b].fuzzy_step(bounds, feed[b])
                gpu.assert_close(gl[b], wl, TOL["bf16"], f"fuzzy logits, sequence {b}, step {step}")
        calib = {0: [int(t) for t in toks[0, 4:10]], 1: [int(toks[1, 4])], 3: [int(t) for t in toks[3, 4:7]]}
        gt, gl = g.calibrate(calib, all_rows=True)
        for b, t in calib.items():
            wl = seqs[b].calibrate(t, all_rows=True)
            gpu.assert_close(gl[b], wl, TOL["bf16"], f"calibration logits, sequence {b}")
        p, f = g.lens()
        assert [int(x) for x in p] == [s.precise for s in seqs] and [int(x) for x in f] == [s.fuzzy for s in seqs]
        assert seqs[2].fuzzy == 3 and seqs[0].fuzzy == 0
        feed = {b: int(toks[b, 12]) for b in range(4)}
        gt, gl = g.draft_step(feed)
        for b in range(4):
            gpu.assert_close(gl[b], seqs[b].fuzzy_step(bounds, feed[b]), TOL["bf16"])
    finally:
        g.close()


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_batch16_ragged_contexts(oracle, gpu, dtype):
    """Sixteen sequences whose contexts run from 1 slot to several split-KV chunks in one launch: every
    column gets its own number of chunks (one for the short ones) and its own ragged last batch."""
    cfg = synth.model_shape("tiny", dtype=dtype)
    w = synth.make_weights(cfg, 570)
    rng = np.random.Generator(np.random.Philox(key=[571, 0]))
    ctxs = [1, 2, 31, 33, 63, 64, 65, 255, 256, 257] + [int(x) for x in rng.integers(258, 1500, 6)]
    max_ctx = 1536
    model = oracle.Model(cfg, w, max_ctx)
    seqs = [oracle.Sequence(model) for _ in ctxs]
    g = gpu.GpuDrafter(cfg, w, max_batch=16, max_ctx=max_ctx, max_calib=4)
    bounds = np.array([0, 1, 3, 4], np.int32)
    try:
        g.set_groups(bounds)
        for b, n in enumerate(ctxs):
            k, v = synth.make_kv_prefix(cfg, 572, n, seq=b)
            seqs[b].import_kv(k, v); g.import_kv(b, k, v)
        toks = synth.make_tokens(573, 16 * 8, cfg["vocab"]).reshape(16, 8)
        for step in range(3):
            feed = {b: int(toks[b, step]) for b in range(16)}
            gt, gl = g.draft_step(feed)
            for b in range(16):
                wl = seqs[b].fuzzy_step(bounds, feed[b])
                gpu.assert_close(gl[b], wl, TOL[dtype], f"fuzzy logits, sequence {b} (context {ctxs[b]}), step {step}")
        # calibration of a few of them (4 + 4 + 4 + 4 columns), the others keep their fuzzy slots
        calib = {b: [int(t) for t in toks[b, 4:8]] for b in (0, 5, 9, 15)}
        gt, gl = g.calibrate(calib, all_rows=True)
        for b, t in calib.items():
            wl = seqs[b].calibrate(t, all_rows=True)
            gpu.assert_close(gl[b], wl, TOL[dtype], f"calibration logits, sequence {b}")
        p, f = g.lens()
        assert [int(x) for x in p] == [s.precise for s in seqs] and [int(x) for x in f] == [s.fuzzy for s in seqs]
    finally:
        g.close()


@pytest.mark.parametrize("shape,dtype", [("tiny", "fp32"), ("tiny", "bf16"), ("tiny_qwen", "bf16")])
def test_maximum_context_filled_to_the_last_slot(oracle, gpu, shape, dtype):
    """The library's largest context (65 536 slots: 64 split-KV chunks of 1024) on small models: a synthetic prefix,
    a 9-token calibration, fuzzy steps, a 4-wide tree level whose last node takes slot 65 535, then every further
    call is refused with ECAPACITY and leaves the lengths alone."""
    import paper_2502_02493_amd as es
    cfg = synth.model_shape(shape, dtype=dtype)
    w = synth.make_weights(cfg, 540)
    max_ctx, tol = 65536, TOL[dtype]
    bounds = groups(es, cfg, 2, "packed")
    so = oracle.Sequence(oracle.Model(cfg, w, max_ctx))
    g = gpu.GpuDrafter(cfg, w, max_batch=1, max_ctx=max_ctx, max_calib=16)
    try:
        g.set_groups(bounds)
        n0 = max_ctx - 9 - 3 - 4
        k, v = synth.make_kv_prefix(cfg, 541, n0)
        so.import_kv(k, v); g.import_kv(0, k, v)
        toks = [int(t) for t in synth.make_tokens(542, 32, cfg["vocab"])]
        wl = so.calibrate(toks[:9], all_rows=True)
        _, gl = g.calibrate({0: toks[:9]}, all_rows=True)
        gpu.assert_close(gl[0], wl, tol, "9-token calibration behind 65 520 slots")
        # the calibration again after a chain of fuzzy steps was dropped
        for t in toks[9:12]:
            gpu.assert_close(g.draft_step({0: t})[1][0], so.fuzzy_step(bounds, t), tol, "fuzzy step")
        es.easyspec_truncate(g.ctx, 0, n0 + 9); so.set_lens(n0 + 9, 0)
        for t in toks[12:15]:
            gpu.assert_close(g.draft_step({0: t})[1][0], so.fuzzy_step(bounds, t), tol, "fuzzy step")
        es.easyspec_truncate(g.ctx, 0, n0 + 9); so.set_lens(n0 + 9, 0)
        wl = so.calibrate(toks[15:18], all_rows=True)
        _, gl = g.calibrate({0: toks[15:18]}, all_rows=True)
        gpu.assert_close(gl[0], wl, tol, "3-token calibration")
        wl = so.fuzzy_tree_step(bounds, toks[18:22], [-1, -1, -1, -1])
        _, gl = g.draft_tree_step({0: (toks[18:22], [-1, -1, -1, -1])})
        gpu.assert_close(gl[0], wl, tol, "tree level that fills the context")
        p, f = g.lens()
        assert int(p[0]) + int(f[0]) == max_ctx == so.precise + so.fuzzy
        for call in (lambda: g.draft_tree_step({0: ([1], [0])}), lambda: g.calibrate({0: toks[:5]})):
            with pytest.raises(es.EasySpecError) as e:
                call()
            assert e.value.code == es.EASYSPEC_ECAPACITY
        p2, f2 = g.lens()
        assert (int(p2[0]), int(f2[0])) == (int(p[0]), int(f[0]))
        gk, gv = g.export_kv(0, max_ctx)
        assert gpu.rel_l2(gk[:, :, n0:], so.K[:, :, n0:]) < (4e-3 if dtype == "bf16" else tol)
        assert gpu.rel_l2(gv[:, :, n0:], so.V[:, :, n0:]) < (4e-3 if dtype == "bf16" else tol)
    finally:
        g.close()


_FULL = {}


def full_weights(shape):
    """Full-size random-init weights, drawn once per shape for all tests of this module (16 GB of host
    memory each; the oracle and the loader only keep references)."""
    if shape not in _FULL:
        _FULL.clear()                      # one shape at a time
        print(f"drawing {shape} weights ...", flush=True)
        _FULL[shape] = synth.make_weights(synth.model_shape(shape), 2025)
    return _FULL[shape]


def compare_full(gpu, got, want_pair, want_plain, what):
    """Full-size logits against both oracles: the one that carries activations like the kernels (tight),
    and the plain one (bf16 weights and cache only) at the bar required of a bf16 model."""
    e1 = gpu.assert_close(got, want_pair, gpu.FULL_SIZE_TOL, what)
    e2 = gpu.assert_close(got, want_plain, gpu.PLAIN_TOL, what + " (plain oracle)")
    print(f"{what}: rel-L2 {e1:.2e}; against the plain oracle {e2:.2e}", flush=True)


def full_size_sampled(oracle, gpu, shape, ctx_len, sizes, want_bounds=None, tree_width=0, calib_tokens=6):
    """A benchmark configuration itself (full depth, aligned sets): one calibration of `calib_tokens`
    tokens, then for each layer-parallel size in `sizes` two fuzzy steps from the same calibrated state,
    all checked against the oracle in both of its modes; optionally one tree level of the given width on
    top (the calibration is redone first, so the chain's fuzzy slots are gone)."""
    import paper_2502_02493_amd as es
    cfg = synth.model_shape(shape)
    w = full_weights(shape)
    pair = oracle.Sequence(oracle.Model(cfg, w, ctx_len + 48))
    plain = oracle.Sequence(oracle.Model(cfg, w, ctx_len + 48).set_rounding(oracle.ACT_PLAIN, True))
    g = gpu.GpuDrafter(cfg, w, max_batch=1, max_ctx=ctx_len + 48, max_calib=16)
    stats = [0, 0]
    try:
        k, v = synth.make_kv_prefix(cfg, 2026, ctx_len)
        pair.import_kv(k, v); plain.import_kv(k, v); g.import_kv(0, k, v)
        calib = [int(t) for t in synth.make_tokens(2027, calib_tokens, cfg["vocab"])]
        print("oracle calibration ...", flush=True)
        wl, wp = pair.calibrate(calib, all_rows=False), plain.calibrate(calib, all_rows=False)
        gt, gl = g.calibrate({0: calib}, all_rows=False)
        compare_full(gpu, gl[0], wl, wp, f"{calib_tokens}-token calibration")
        tok0 = check_ids(oracle, "bf16", gt[0], wl, stats)
        P = pair.precise
        for N in sizes:
            bounds = groups(es, cfg, N)
            if want_bounds is not None and N == sizes[0]:
                assert list(bounds) == want_bounds
            assert int(np.max(np.diff(bounds))) == min(N, cfg["n_layers"] - 2)
            g.set_groups(bounds)
            es.easyspec_truncate(g.ctx, 0, P); pair.set_lens(P, 0); plain.set_lens(P, 0)
            tok = tok0
            for step in range(2):
                wl, wp = pair.fuzzy_step(bounds, tok), plain.fuzzy_step(bounds, tok)
                gtok, glog = g.draft_step({0: tok})
                compare_full(gpu, glog[0], wl, wp, f"N={N} fuzzy step {step}")
                tok = check_ids(oracle, "bf16", gtok[0], wl, stats)
        assert stats[0] >= 2, stats
        if tree_width:
            pair.calibrate([tok]); plain.calibrate([tok])
            g.calibrate({0: [tok]}, all_rows=False)
            toks = [int(t) for t in synth.make_tokens(2028, tree_width, cfg["vocab"])]
            print("oracle tree level ...", flush=True)
            wl, wp = pair.fuzzy_tree_step(bounds, toks, [-1] * tree_width), plain.fuzzy_tree_step(bounds, toks, [-1] * tree_width)
            _, gl = g.draft_tree_step({0: (toks, [-1] * tree_width)})
            compare_full(gpu, gl[0], wl, wp, f"{tree_width}-wide tree level")
    finally:
        g.close()


def test_full_size_llama3_8b_sampled(oracle, gpu):
    """32 layers, context 2048, sets of 4, 6-token calibration; then a tree level of width 8 (matrix-core
    attention at full size)."""
    full_size_sampled(oracle, gpu, "llama3_8b", 2048, [4], [0, 1, 4, 8, 12, 16, 20, 24, 28, 31, 32], tree_width=8)


def test_full_size_llama3_8b_long_calibration_sampled(oracle, gpu):
    """The calibration-dominant configuration: 32 layers, context 8192, a 9-token calibration (more than 8
    columns: two activation fragments per weight tile, matrix-core attention over 9 columns), then fuzzy
    steps and a 4-wide tree level (the vector kernel with the tree mask at full size)."""
    full_size_sampled(oracle, gpu, "llama3_8b", 8192, [4], tree_width=4, calib_tokens=9)


def test_full_size_llama3_8b_batch4_long_contexts(oracle, gpu):
    """The long-context batched configuration at full depth: 32 layers, aligned sets of 4, four sequences
    with contexts 4096 / 8191 / 16367 / 32705 (ragged against every tile) in one fuzzy step — the launch
    sequence bench.py times — and then a calibration of two of them.  The oracle's sequences are
    independent, so it follows one sequence at a time (the longest holds 8.6 GB of float32 cache)."""
    import gc
    import paper_2502_02493_amd as es
    cfg = synth.model_shape("llama3_8b")
    w = full_weights("llama3_8b")
    ctxs = [4096, 8191, 16367, 32705]
    bounds = groups(es, cfg, 4)
    assert list(bounds) == [0, 1, 4, 8, 12, 16, 20, 24, 28, 31, 32]
    g = gpu.GpuDrafter(cfg, w, max_batch=4, max_ctx=32768, max_calib=6)
    try:
        g.set_groups(bounds)
        toks = synth.make_tokens(2032, 64, cfg["vocab"]).reshape(4, 16)
        feed = {b: int(toks[b, 0]) for b in range(4)}
        calib = {0: [int(t) for t in toks[0, 4:10]], 3: [int(t) for t in toks[3, 4:7]]}
        want = {}
        for b, n in enumerate(ctxs):
            print(f"sequence {b}: {n} slots of prefix, oracle fuzzy step ...", flush=True)
            k, v = synth.make_kv_prefix(cfg, 2031, n, seq=b)
            g.import_kv(b, k, v)
            so = oracle.Sequence(oracle.Model(cfg, w, n + 16))
            so.import_kv(k, v)
            del k, v
            want[b] = [so.fuzzy_step(bounds, feed[b])]
            if b in calib:
                want[b].append(so.calibrate(calib[b], all_rows=False))
            del so
            gc.collect()
        gt, gl = g.draft_step(feed)
        for b in range(4):
            err = gpu.assert_close(gl[b], want[b][0], gpu.FULL_SIZE_TOL, f"fuzzy logits, sequence {b} ({ctxs[b]} slots)")
            print(f"sequence {b} ({ctxs[b]} slots): fuzzy step rel-L2 {err:.2e}", flush=True)
            wid, margin = oracle.argmax(want[b][0], with_margin=True)
            if margin > MARGIN["bf16"] * float(np.std(want[b][0])):
                assert int(gt[b]) == wid
        gt, gl = g.calibrate(calib, all_rows=False)
        for b in calib:
            err = gpu.assert_close(gl[b], want[b][1], gpu.FULL_SIZE_TOL, f"calibration logits, sequence {b}")
            print(f"sequence {b}: {len(calib[b])}-token calibration rel-L2 {err:.2e}", flush=True)
        p, f = g.lens()
        assert [int(x) for x in p] == [4096 + 6, 8191, 16367, 32705 + 3] and [int(x) for x in f] == [0, 1, 1, 0]
    finally:
        g.close()


def test_full_size_qwen2_7b_sampled(oracle, gpu):
    """28 layers, context 4096, 7 query heads per KV head, QKV bias, layer-parallel sizes 4, 2 and 7 of the
    configuration's sweep (N = 7: sets 0 | 1-6 | 7-13 | 14-20 | 21-26 | 27, the 7-layer stacked launches
    at d = 3584)."""
    full_size_sampled(oracle, gpu, "qwen2_7b", 4096, [4, 2, 7])
