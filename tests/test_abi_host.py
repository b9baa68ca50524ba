"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and its host-side logic (strategy helper, host greedy acceptance, argument checks) is right.
No kernel is launched here."""
import itertools
import os
import re

import numpy as np
import pytest

import easyspec_synth as synth
import paper_2502_02493_amd as es

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _headers():
    inc = os.path.join(ROOT, "include")
    return "\n".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))


def test_library_exports_every_declared_symbol():
    header = _headers()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(easyspec_[a-z_]+)\s*\(", header))
    assert declared, "no declarations found"
    lib = es.load_library()
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in easyspec.h but not exported"
    assert declared == set(es.EXPORTS), declared ^ set(es.EXPORTS)


def test_header_constants_match_binding():
    header = _headers()
    for name in ("EASYSPEC_OK", "EASYSPEC_EINVAL", "EASYSPEC_ECAPACITY", "EASYSPEC_ESTATE", "EASYSPEC_EHIP",
                 "EASYSPEC_DTYPE_F32", "EASYSPEC_DTYPE_BF16", "EASYSPEC_POLICY_ALIGNED", "EASYSPEC_POLICY_PACKED",
                 "EASYSPEC_MAX_BATCH", "EASYSPEC_MAX_CALIB_TOKENS", "EASYSPEC_MAX_SET", "EASYSPEC_OP_QKV",
                 "EASYSPEC_OP_ATTN", "EASYSPEC_OP_OPROJ", "EASYSPEC_OP_GATEUP", "EASYSPEC_OP_DOWN", "EASYSPEC_OP_HEAD", "EASYSPEC_OP_ALL",
                 "EASYSPEC_MAX_TREE_WIDTH", "EASYSPEC_MAX_TREE_NODES", "EASYSPEC_MAX_CHUNKS", "EASYSPEC_PARALLEL_ATTENTION",
                 "EASYSPEC_PARALLEL_FULL_LAYER"):
        m = re.search(rf"#define\s+{name}\s+\(?(-?\d+)\)?", header)
        assert m, name
        assert int(m.group(1)) == getattr(es.binding, name), name


def test_method_header_declares_no_instrumentation():
    """easyspec.h is the boundary of the method; timing, probes, host models and poisoning live in
    easyspec_instrument.h."""
    core = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "easyspec.h")).read(), flags=re.S)
    for name in ("easyspec_profile_begin", "easyspec_profile_end", "easyspec_stream_read", "easyspec_attention_cut",
                 "easyspec_weight_walk", "easyspec_poison_workspaces"):
        assert name not in core, name
    for name in ("easyspec_draft_step", "easyspec_calibrate", "easyspec_greedy_accept", "easyspec_accept", "easyspec_draft_tree_step"):
        assert name in core, name


def test_default_groups_matches_paper_table_and_oracle(oracle):
    """The product's own helper against the rows printed in Sec. 3.1.1 and against the oracle's
    independently written helper over a sweep of shapes."""
    def sets(bounds):
        return [f"{a}" if b - a == 1 else f"{a}-{b - 1}" for a, b in zip(bounds[:-1], bounds[1:])]
    rows = [l for l in open(os.path.join(ROOT, "tests", "golden", "layer_parallel_strategies.txt"))
            if l.strip() and l[0] != "#"]
    for row in rows:
        left, head, tail = [p.split() for p in row.split("|")]
        L, N = int(left[0]), int(left[1])
        pol = es.EASYSPEC_POLICY_ALIGNED if left[2] == "aligned" else es.EASYSPEC_POLICY_PACKED
        got = sets(es.easyspec_default_groups(L, N, pol))
        assert got[: len(head)] == head and got[-len(tail):] == tail
    for L, N in itertools.product(range(1, 40), range(1, 9)):
        for pol, name in ((0, "aligned"), (1, "packed")):
            b = es.easyspec_default_groups(L, N, pol)
            assert list(b) == list(oracle.default_groups(L, N, name)), (L, N, name)
            assert b[0] == 0 and b[-1] == L and np.all(np.diff(b) >= 1) and np.all(np.diff(b) <= max(N, 1))
            if L >= 3:
                assert b[1] == 1 and b[-2] == L - 1          # first and last layer are sets of their own


def test_default_groups_rejects_bad_arguments():
    for args in ((0, 4, 0), (8, 0, 0), (8, 4, 2), (-1, 4, 0)):
        with pytest.raises(es.EasySpecError) as e:
            es.easyspec_default_groups(*args)
        assert e.value.code == es.EASYSPEC_EINVAL


def test_greedy_accept_host_path(oracle):
    """Host loop of the C ABI against the oracle on every draft/target pair for gamma <= 3 over
    three symbols, batched, plus gamma = 0 (nothing drafted: the bonus is the only token)."""
    for gamma in (1, 2, 3):
        drafts = list(itertools.product(range(3), repeat=gamma))
        targets = list(itertools.product(range(3), repeat=gamma + 1))
        pairs = list(itertools.product(drafts, targets))
        d = np.array([p[0] for p in pairs], np.int32)
        t = np.array([p[1] for p in pairs], np.int32)
        acc, bonus = np.zeros(len(pairs), np.int32), np.zeros(len(pairs), np.int32)
        es.easyspec_greedy_accept_host(d, t, len(pairs), gamma, acc, bonus)
        for i, (dd, tt) in enumerate(pairs):
            assert (int(acc[i]), int(bonus[i])) == oracle.greedy_accept(dd, tt)
    acc, bonus = np.zeros(2, np.int32), np.zeros(2, np.int32)
    es.easyspec_greedy_accept_host(np.zeros(0, np.int32), np.array([[7], [9]], np.int32), 2, 0, acc, bonus)
    assert list(acc) == [0, 0] and list(bonus) == [7, 9]
    with pytest.raises(es.EasySpecError):
        es.easyspec_greedy_accept_host(None, np.zeros(2, np.int32), 1, 1, acc, bonus)
    with pytest.raises(es.EasySpecError):
        es.easyspec_greedy_accept_host(np.zeros(1, np.int32), np.zeros(2, np.int32), 0, 1, acc, bonus)


def test_greedy_accept_device_entry_refuses_host_arrays():
    """The device entry point never falls back to a host loop: host arrays (or no device at all) are an
    error, whatever the stream handle is; the null stream is a stream like any other."""
    acc, bonus = np.zeros(1, np.int32), np.zeros(1, np.int32)
    for stream in (None, 0):
        with pytest.raises(es.EasySpecError) as e:
            es.easyspec_greedy_accept(np.zeros(1, np.int32), np.zeros(2, np.int32), 1, 1, acc, bonus, stream)
        assert e.value.code in (es.EASYSPEC_EINVAL, es.EASYSPEC_EHIP)
    assert list(acc) == [0] and list(bonus) == [0]


def test_create_rejects_bad_shapes_before_touching_the_device():
    import easyspec_synth as synth
    good = synth.model_shape("tiny")
    bad = [dict(head_dim=48), dict(d_model=250), dict(d_ffn=1000), dict(n_q_heads=6, n_kv_heads=2, d_model=384),
           dict(n_kv_heads=3), dict(n_layers=0), dict(vocab=0), dict(rope_theta=0.0)]
    for over in bad:
        with pytest.raises(es.EasySpecError) as e:
            es.easyspec_create(es.make_config(dict(good, **over), 1, 64, 4))
        assert e.value.code == es.EASYSPEC_EINVAL, over
    for mb, mc, mt in ((0, 64, 4), (17, 64, 4), (1, 0, 4), (1, 64 * 1024 + 1, 4), (1, 64, 0), (1, 64, 17)):
        with pytest.raises(es.EasySpecError) as e:
            es.easyspec_create(es.make_config(good, mb, mc, mt))
        assert e.value.code == es.EASYSPEC_EINVAL


def test_no_cpu_fallback():
    """Without a HIP device the library refuses to create a context (EASYSPEC_EHIP): there is no
    CPU path that a parity test could silently run on."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible here")
    import easyspec_synth as synth
    with pytest.raises(es.EasySpecError) as e:
        es.easyspec_create(es.make_config(synth.model_shape("tiny"), 1, 64, 4))
    assert e.value.code == es.EASYSPEC_EHIP
    assert "no HIP device" in str(e.value)


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2502_02493_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, f"{f} mentions the oracle"
    assert "paper_2502_02493_amd" not in open(os.path.join(ROOT, "oracle", "easyspec_oracle.py")).read()
    assert "paper_2502_02493_amd" not in open(os.path.join(ROOT, "oracle", "easyspec_oracle.c")).read()


def test_accept_rejects_bad_arguments_on_the_host():
    """Argument checks of the sampling acceptance come before any device work."""
    a = np.zeros(8, np.float32)
    i = np.zeros(8, np.int32)
    w = np.zeros(64, np.float64)
    ok = dict(draft=i, draft_logits=a, target_logits=a, r=a, u=a, batch=1, gamma=1, vocab=2, temperature=1.0,
              accept_len=i, bonus=i, workspace=w)
    for over in (dict(temperature=0.0), dict(temperature=-1.0), dict(temperature=float("inf")), dict(batch=0), dict(gamma=-1),
                 dict(gamma=65), dict(vocab=0), dict(target_logits=None), dict(workspace=None), dict(draft=None), dict(u=None)):
        with pytest.raises(es.EasySpecError) as e:
            es.easyspec_accept(**dict(ok, **over))
        assert e.value.code == es.EASYSPEC_EINVAL, over
    assert es.easyspec_accept_workspace_bytes(4, 5, 1000) >= 4 * (11 * 16 + 1000 * 8)
    assert es.easyspec_accept_workspace_bytes(0, 5, 1000) == -1
    assert es.easyspec_accept_workspace_bytes(1, 5, 0) == -1
    import torch
    if not torch.cuda.is_available():
        with pytest.raises(es.EasySpecError) as e:      # valid arguments, no device: refused, never computed on the CPU
            es.easyspec_accept(**ok)
        assert e.value.code == es.EASYSPEC_EHIP


def test_stream_read_rejects_bad_arguments_on_the_host():
    a = np.zeros(64, np.float32)
    for buf, n, sink in ((None, 64, a), (a, 64, None), (a, 0, a), (a, 24, a), (a, -16, a)):
        with pytest.raises(es.EasySpecError) as e:
            es.easyspec_stream_read(buf, n, sink)
        assert e.value.code == es.EASYSPEC_EINVAL
    assert es.easyspec_stream_read_sink_floats() >= 1


def test_attention_cut_gives_every_slot_to_exactly_one_wave():
    """The split-KV cut of the vector attention kernel, evaluated on the host with the kernels' own index
    functions: whatever the mix of context lengths, the chunks of a column tile its context in order, the
    waves of a chunk tile the chunk, chunk counts respect the partial buffers, and contexts that all fit
    one piece are not split."""
    import paper_2502_02493_amd as es
    rng = np.random.default_rng(77)
    shapes = [("llama3_8b", "bf16"), ("qwen2_7b", "bf16"), ("tiny", "fp32"), ("tiny", "bf16"), ("tiny_qwen", "bf16")]
    special = [1, 2, 7, 8, 9, 31, 32, 33, 255, 256, 257, 511, 513, 2047, 2048, 2049, 2055, 4097, 8191, 32768, 65535, 65536]
    cases = 0
    for shape, dtype in shapes:
        cfg = es.make_config(synth.model_shape(shape, dtype=dtype), 16, 65536, 16)
        for trial in range(60):
            n_cols = int(rng.integers(1, 17))
            if trial % 3 == 0:
                lens = [int(rng.choice(special)) for _ in range(n_cols)]
            elif trial % 3 == 1:
                base = int(rng.choice(special))
                lens = [max(1, min(65536, base + i)) for i in range(n_cols)]          # a calibration: consecutive lengths
            else:
                lens = [int(x) for x in np.exp(rng.uniform(0, np.log(65536), n_cols)).astype(int).clip(1, 65536)]
            for n_set in (1, 3, 4, 8):
                nwv, n_chunks, ranges = es.easyspec_attention_cut(cfg, lens, n_set)
                assert nwv in (4, 8)
                if max(lens) <= 256:
                    assert nwv == 8 and all(n == 1 for n in n_chunks)
                for i, n in enumerate(lens):
                    assert 1 <= n_chunks[i] <= es.EASYSPEC_MAX_CHUNKS
                    at = 0
                    for ch in range(n_chunks[i]):
                        for w in range(nwv):
                            lo, hi = (int(x) for x in ranges[i, ch, w])
                            assert lo == at or hi == lo, (shape, lens, n_set, i, ch, w, lo, hi, at)   # in order, no gap
                            assert hi >= lo
                            if hi > lo:
                                at = hi
                        assert not ranges[i, ch, nwv:].any()
                    assert at == n, (shape, lens, n_set, i, at)
                    assert not ranges[i, n_chunks[i]:].any()
                cases += 1
    assert cases == len(shapes) * 60 * 4


def test_attention_cut_rejects_bad_arguments():
    import paper_2502_02493_amd as es
    cfg = es.make_config(synth.model_shape("tiny", dtype="fp32"), 4, 512, 8)
    for lens, n_set in (([0], 1), ([513], 1), ([5] * 17, 1), ([5], 0), ([5], 9)):
        with pytest.raises(es.EasySpecError):
            es.easyspec_attention_cut(cfg, lens, n_set)


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: `bench.py --gpus 2` must say so and exit without touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


# ---------------------------------------------------------------------------- the weight stream's index arithmetic

WEIGHT_OPS = ("EASYSPEC_OP_QKV", "EASYSPEC_OP_OPROJ", "EASYSPEC_OP_GATEUP", "EASYSPEC_OP_DOWN", "EASYSPEC_OP_HEAD")


def check_walk(cfg, op, n_cols, k, full=False):
    """Every piece a launch reads lies inside the packed matrices of its layers, reaches their last piece, and
    every k-tile of every row tile is read exactly once (a missing last unit of a two-unit workgroup is
    re-read on purpose); every activation fragment lies inside its operand slot."""
    r = es.easyspec_weight_walk(cfg, getattr(es, op), n_cols, k, full)
    what = (op, n_cols, k, full, r)
    assert r["w_out_of_range"] == 0 and 0 <= r["w_max"] == r["w_pieces"] - 1, what
    assert r["x_out_of_range"] == 0 and 0 <= r["x_max"] < r["x_slot_elems"], what
    assert r["missed_tiles"] == 0 and r["repeated_tiles"] == 0 and r["uncovered_pieces"] == 0, what
    if r["units_per_wg"] == 1:
        assert r["reread_tiles"] == 0, what
    assert r["grid"] >= 1 and 1 <= r["waves"] <= 16 and r["fragments"] == (2 if cfg.dtype == es.EASYSPEC_DTYPE_BF16 and n_cols > 8 else 1), what
    return r


@pytest.mark.parametrize("shape,dtype", [("tiny", "fp32"), ("tiny", "bf16"), ("tiny_qwen", "fp32"), ("tiny_qwen", "bf16")])
def test_weight_stream_index_arithmetic_small_shapes(monkeypatch, shape, dtype):
    """Host walk of every weight-streaming launch shape of the small models: all column counts, set sizes,
    both parallel modes, forced wave counts (including counts that do not divide K), forced tile heights and
    forced two-unit workgroups.  A wrong tile-to-wave assignment (a skipped or doubled k-tile), a wrong clamp
    of the last unit or a lane piece outside its fragment shows up here, on the CPU, before any launch."""
    base = synth.model_shape(shape, dtype=dtype)
    cfg = es.make_config(base, 2, 128, 16)
    n = 0
    for op in WEIGHT_OPS:
        for n_cols in range(1, 17):
            for k in (1, 2, 3, base["n_layers"]):
                check_walk(cfg, op, n_cols, k)
                n += 1
                if op in ("EASYSPEC_OP_OPROJ", "EASYSPEC_OP_GATEUP", "EASYSPEC_OP_DOWN"):
                    check_walk(cfg, op, n_cols, k, full=True)
    assert n == 5 * 16 * 4
    for env in ("EASYSPEC_NW_QKV", "EASYSPEC_NW_O", "EASYSPEC_NW_GU", "EASYSPEC_NW_DOWN", "EASYSPEC_NW_HEAD"):
        for nw in (1, 2, 3, 5, 6, 7, 8, 11, 16):
            monkeypatch.setenv(env, str(nw))
            for op in WEIGHT_OPS:
                for n_cols in (1, 5, 12):
                    check_walk(cfg, op, n_cols, 2)
        monkeypatch.delenv(env)
    for pair in ("0", "1"):
        monkeypatch.setenv("EASYSPEC_PAIR_TILES", pair)
        for rows in (13, 14, 15, 16):
            monkeypatch.setenv("EASYSPEC_TILE_ROWS", str(rows))
            for qrows in (8, 12, 16):
                monkeypatch.setenv("EASYSPEC_QKV_TILE_ROWS", str(qrows))
                for op in WEIGHT_OPS:
                    for n_cols in (1, 9, 16):
                        r = check_walk(cfg, op, n_cols, 3)
                        if dtype == "bf16" and n_cols > 8 and op != "EASYSPEC_OP_DOWN":
                            assert r["units_per_wg"] == (2 if pair == "1" else 1)


@pytest.mark.parametrize("shape", ["llama3_8b", "qwen2_7b"])
def test_weight_stream_index_arithmetic_benchmark_shapes(shape):
    """The same walk at the two benchmark shapes with the launch shapes the library picks there (14-row gate/up
    tiles and 12-pair QKV tiles at the 8B width, seven waves in the down projection, two-unit workgroups in
    two-fragment passes where they fill the CUs), for the set sizes of the benchmark strategies."""
    base = synth.model_shape(shape)
    cfg = es.make_config(base, 4, 32768, 16)
    seen_two_units = False
    for op in WEIGHT_OPS:
        for n_cols, k in ((1, 1), (1, 3), (1, 4), (1, 7), (4, 4), (6, 1), (9, 1), (12, 4), (16, 8)):
            r = check_walk(cfg, op, n_cols, k)
            seen_two_units = seen_two_units or r["units_per_wg"] == 2
    assert seen_two_units
    r = check_walk(cfg, "EASYSPEC_OP_DOWN", 1, 1)
    assert r["waves"] == (7 if shape == "llama3_8b" else 8) and r["grid"] == base["d_model"] // 16
    r = check_walk(cfg, "EASYSPEC_OP_GATEUP", 1, 1)
    assert r["tile_rows"] == (14 if shape == "llama3_8b" else 16)
    for op in ("EASYSPEC_OP_OPROJ", "EASYSPEC_OP_GATEUP", "EASYSPEC_OP_DOWN"):
        check_walk(cfg, op, 1, 4, full=True)


def test_weight_walk_rejects_bad_arguments():
    cfg = es.make_config(synth.model_shape("tiny"), 1, 64, 16)
    for args in ((es.EASYSPEC_OP_ATTN, 1, 1), (es.EASYSPEC_OP_QKV, 0, 1), (es.EASYSPEC_OP_QKV, 17, 1), (es.EASYSPEC_OP_QKV, 1, 0),
                 (es.EASYSPEC_OP_QKV, 1, 9), (es.EASYSPEC_OP_QKV, 1, 5), (es.EASYSPEC_OP_ALL, 1, 1)):
        with pytest.raises(es.EasySpecError) as e:
            es.easyspec_weight_walk(cfg, *args)
        assert e.value.code == es.EASYSPEC_EINVAL


def test_attention_stage_walk_delivers_every_k_piece_to_its_mfma_operand():
    """The passage of a batch of K rows through a wave's LDS into MFMA A fragments (vector attention with scores
    from the matrix cores), walked on the host with the kernel's own index functions: every stored piece has a
    place of its own inside the wave's 8 KB, every fetch returns the piece its operand position needs, the score
    of a slot comes out where that slot's V row sits, and no quarter-wave meets a bank group twice."""
    import paper_2502_02493_amd as es
    for n_loads in (2, 8):
        rep = es.easyspec_attention_stage_walk(n_loads)
        assert rep["stored"] == rep["distinct_places"] == 64 * n_loads
        assert rep["highest_place"] <= rep["places"] == 512
        tiles = (n_loads + 3) // 4
        assert rep["fetched"] + rep["unused_rows"] == 64 * 4 * tiles
        assert rep["fetched"] == 16 * n_loads * 4          # every piece of every row of the batch, once
        assert rep["wrong_piece"] == 0
        assert rep["misplaced_scores"] == 0
        assert rep["bank_conflicts"] == 0
    for bad in (0, 1, 4, 16):
        with pytest.raises(es.EasySpecError) as e:
            es.easyspec_attention_stage_walk(bad)
        assert e.value.code == es.EASYSPEC_EINVAL
