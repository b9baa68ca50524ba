"""CPU pins of the oracle against what the paper and the mathematics fix.

Each test names the mistake it is there to catch.  None of them compares the oracle with
itself through the same code path: the library decoder (tests/hf_ref.py), closed forms,
brute force, or two separately written oracle paths that the paper says must coincide.
"""
import itertools
import os

import numpy as np
import pytest

import easyspec_synth as synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def as_f64(w):
    """Synthetic parameters as float64 (bf16 bit patterns widened)."""
    def conv(a):
        return synth.bf16_bits_to_f32(a).astype(np.float64) if a.dtype == np.uint16 else a.astype(np.float64)
    out = {k: conv(v) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: conv(v) for k, v in lw.items()} for lw in w["layers"]]
    return out


@pytest.fixture(scope="module")
def tiny(oracle):
    cfg = synth.model_shape("tiny")
    w = synth.make_weights(cfg, seed=1)
    return cfg, w, oracle.Model(cfg, w, max_ctx=64)


@pytest.fixture(scope="module")
def tiny_qwen(oracle):
    cfg = synth.model_shape("tiny_qwen")
    w = synth.make_weights(cfg, seed=2)
    return cfg, w, oracle.Model(cfg, w, max_ctx=64)


# ---------------------------------------------------------------------------- primitives

def test_bf16_round_matches_torch(oracle):
    """Rounding helper vs the library's float32->bfloat16 cast (ties, both signs, tiny values)."""
    import torch
    rng = np.random.default_rng(0)
    xs = np.concatenate([rng.standard_normal(2000).astype(np.float32) * 3,
                         np.float32([1 + 2**-8, 1 + 3 * 2**-8, -(1 + 2**-8), 2**-20 * (1 + 2**-8), 0.0, 255.5, 256.5]),
                         rng.standard_normal(200).astype(np.float32) * 1e-6])
    want = torch.from_numpy(xs).to(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([oracle.bf16_round(float(x)) for x in xs])
    assert np.array_equal(got, want)
    assert np.array_equal(synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(xs)).astype(np.float64), want)


def test_matvec_vs_numpy(oracle):
    """Dropped bias, transposed operand or wrong widening of bf16 bits."""
    rng = np.random.default_rng(1)
    w = rng.standard_normal((37, 53)).astype(np.float32)
    x = rng.standard_normal(53)
    b = rng.standard_normal(37).astype(np.float32)
    assert np.allclose(oracle.matvec(w, x, b), w.astype(np.float64) @ x + b, rtol=1e-13, atol=1e-13)
    assert np.allclose(oracle.matvec(w, x, b, scale=0.37), 0.37 * (w.astype(np.float64) @ x) + b, rtol=1e-13, atol=1e-13)
    wb = synth.f32_to_bf16_bits(w)
    assert np.allclose(oracle.matvec(wb, x), synth.bf16_bits_to_f32(wb).astype(np.float64) @ x, rtol=1e-13, atol=1e-13)


def test_rmsnorm_closed_form(oracle):
    """Unit gain: output has mean square 1/(1 + eps/ms); gain scales elementwise; scale invariance."""
    rng = np.random.default_rng(2)
    x = rng.standard_normal(256) * 3.0
    one = np.ones(256, dtype=np.float32)
    y = oracle.rmsnorm(x, one, 1e-6)
    ms = np.mean(x * x)
    assert np.isclose(np.mean(y * y), ms / (ms + 1e-6), rtol=1e-12)
    g = rng.standard_normal(256).astype(np.float32)
    assert np.allclose(oracle.rmsnorm(x, g, 1e-6), y * g, rtol=1e-13)
    assert np.allclose(oracle.rmsnorm(7.0 * x, one, 0.0), oracle.rmsnorm(x, one, 0.0), rtol=1e-12)
    # mean-centred LayerNorm would fail this: a constant vector maps to its sign
    assert np.allclose(oracle.rmsnorm(np.full(8, 5.0), np.ones(8, np.float32), 0.0), np.ones(8))


def test_softmax_silu_library(oracle):
    import scipy.special as sp
    rng = np.random.default_rng(3)
    s = rng.standard_normal(97) * 20
    assert np.allclose(oracle.softmax(s), sp.softmax(s), rtol=1e-13, atol=0)
    for z in (-30.0, -1.0, 0.0, 0.5, 12.0):
        assert np.isclose(oracle.silu(z), z * sp.expit(z), rtol=1e-14, atol=1e-300)


def test_rope_properties(oracle):
    """Position 0 is the identity; norm is preserved; <R_p q, R_s k> depends on p - s only;
    the first pair rotates by exactly `pos` radians (pairing i <-> i + hd/2, frequency 1 at i=0)."""
    rng = np.random.default_rng(4)
    hd, theta = 64, 10000.0
    q, k = rng.standard_normal(hd), rng.standard_normal(hd)
    assert np.array_equal(oracle.rope(q, 0, theta), q)
    assert np.isclose(np.linalg.norm(oracle.rope(q, 1234, theta)), np.linalg.norm(q), rtol=1e-13)
    a = oracle.rope(q, 17, theta) @ oracle.rope(k, 5, theta)
    b = oracle.rope(q, 112, theta) @ oracle.rope(k, 100, theta)
    assert np.isclose(a, b, rtol=1e-11)
    e = np.zeros(hd); e[0] = 1.0
    r = oracle.rope(e, 3, theta)
    assert np.isclose(r[0], np.cos(3.0)) and np.isclose(r[hd // 2], np.sin(3.0))
    # last pair rotates with frequency theta^(-(hd-2)/hd)
    e = np.zeros(hd); e[hd // 2 - 1] = 1.0
    r = oracle.rope(e, 1000, theta)
    ang = 1000 * theta ** (-(hd - 2) / hd)
    assert np.isclose(r[hd // 2 - 1], np.cos(ang)) and np.isclose(r[hd - 1], np.sin(ang))


def test_argmax_lowest_index_on_ties(oracle):
    assert oracle.argmax(np.array([1.0, 5.0, 5.0, 2.0])) == 1
    i, m = oracle.argmax(np.array([0.0, 3.0, 2.5]), with_margin=True)
    assert i == 1 and np.isclose(m, 0.5)


# ---------------------------------------------------------------------------- Alg. 3, greedy

def test_greedy_accept_brute_force(oracle):
    """All draft/target pairs for gamma <= 3 over a 3-symbol vocabulary, against the sequential
    accept/reject scan of Alg. 3 with one-hot distributions (ratio p/p' is 1 or 0)."""
    for gamma in (1, 2, 3):
        for draft in itertools.product(range(3), repeat=gamma):
            for target in itertools.product(range(3), repeat=gamma + 1):
                n = gamma
                for i in range(gamma):
                    ratio = 1.0 if target[i] == draft[i] else 0.0     # p_i(x'_i) / p'_i(x'_i)
                    if 0.5 > ratio:                                    # any r in (0,1) rejects iff ratio == 0
                        n = i
                        break
                bonus = target[n]      # residual max(0, p - p') of one-hots is p itself when they differ
                assert oracle.greedy_accept(draft, target) == (n, bonus)


def test_strategy_table(oracle):
    """Set boundaries against the rows the paper prints (Sec. 3.1.1 table)."""
    def sets(bounds):
        return [f"{a}" if b - a == 1 else f"{a}-{b - 1}" for a, b in zip(bounds[:-1], bounds[1:])]
    rows = [l for l in open(os.path.join(GOLDEN, "layer_parallel_strategies.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 3
    for row in rows:
        left, head, tail = [p.split() for p in row.split("|")]
        L, N, policy = int(left[0]), int(left[1]), left[2]
        got = sets(oracle.default_groups(L, N, policy))
        assert got[: len(head)] == head and got[-len(tail):] == tail, (row, got)
        mid = oracle.default_groups(L, N, policy)
        sizes = np.diff(mid)[len(head):-len(tail)]
        assert np.all(sizes == N)              # the elided middle continues with full N-sets
    # the text rule on the 16-layer model does NOT give the printed row: the reason for two policies
    assert sets(oracle.default_groups(16, 2, "aligned"))[:3] == ["0", "1", "2-3"]


# ---------------------------------------------------------------------------- the decoder itself

@pytest.mark.parametrize("which", ["tiny", "tiny_qwen"])
def test_sequential_matches_library_decoder(oracle, request, which):
    """Alg. 1 through the oracle == an independent library decoder (float64) on the same
    parameters: logits of a prefill, of token-by-token decoding, and every KV entry.
    Catches wrong RoPE pairing/frequency, GQA head mapping, norm placement, SwiGLU order,
    bias handling, residual wiring, transposed weights."""
    from hf_ref import build_hf, hf_prefill, cache_kv
    cfg, w, model = request.getfixturevalue(which)
    hf = build_hf(cfg, as_f64(w))
    toks = synth.make_tokens(5, 12, cfg["vocab"])
    want_logits, cache = hf_prefill(hf, toks)

    s = oracle.Sequence(model)
    got = np.stack([s.sequential_step(t) for t in toks])
    assert rel_l2(got, want_logits) < 1e-6          # float32 KV storage is the only rounding
    for layer in range(cfg["n_layers"]):
        k, v = cache_kv(cache, layer)
        assert rel_l2(s.K[layer, :, :12], k) < 1e-6
        assert rel_l2(s.V[layer, :, :12], v) < 1e-6

    s2 = oracle.Sequence(model)
    got2 = s2.calibrate(toks, all_rows=True)
    assert rel_l2(got2, want_logits) < 1e-6


@pytest.mark.parametrize("which,bounds", [("tiny", [0, 1, 3, 4]), ("tiny", [0, 2, 4]), ("tiny", [0, 4]),
                                          ("tiny_qwen", [0, 1, 4, 5])])
def test_fuzzy_step_matches_library_composition(oracle, request, which, bounds):
    """Alg. 2 with sets larger than one, against the same algorithm composed from the library's
    attention / MLP / norm modules.  The paper prints no number for this quantity; this and the
    invariants below are what pins it."""
    from hf_ref import build_hf, hf_prefill, hf_fuzzy_step
    cfg, w, model = request.getfixturevalue(which)
    hf = build_hf(cfg, as_f64(w))
    toks = synth.make_tokens(6, 9, cfg["vocab"])
    _, cache = hf_prefill(hf, toks[:8])
    want_logits, want_attn = hf_fuzzy_step(hf, cache, toks[8], bounds)

    s = oracle.Sequence(model)
    s.calibrate(toks[:8])
    tap = s.attn_tap()
    got = s.fuzzy_step(bounds, toks[8])
    assert rel_l2(got, want_logits) < 1e-6
    assert rel_l2(tap, want_attn) < 1e-6
    assert (s.precise, s.fuzzy) == (8, 1)
    # and it is a different function from Alg. 1 (otherwise the pin would be vacuous)
    s1 = oracle.Sequence(model)
    s1.calibrate(toks[:8])
    assert rel_l2(s1.sequential_step(toks[8]), want_logits) > 1e-3


def test_group_size_one_is_sequential_bit_exact(oracle, tiny):
    """Alg. 2 with every set of size one is Alg. 1: identical bits in logits, hidden state and KV."""
    cfg, w, model = tiny
    toks = synth.make_tokens(7, 10, cfg["vocab"])
    a, b = oracle.Sequence(model), oracle.Sequence(model)
    a.calibrate(toks[:6]); b.calibrate(toks[:6])
    singles = np.arange(cfg["n_layers"] + 1)
    la, ha = a.sequential_step(toks[6], want_hidden=True)
    lb, hb = b.fuzzy_step(singles, toks[6], want_hidden=True)
    assert np.array_equal(la, lb) and np.array_equal(ha, hb)
    assert np.array_equal(a.K[:, :, :7], b.K[:, :, :7]) and np.array_equal(a.V[:, :, :7], b.V[:, :, :7])
    assert (a.precise, a.fuzzy, b.precise, b.fuzzy) == (7, 0, 6, 1)


def test_fuzzy_attention_reads_set_input_only(oracle, tiny):
    """Within a set, Attnoutput_i and the stored k, v of layer i depend on the set's input h_1
    only: perturbing the MLP of an earlier layer of the same set leaves them unchanged under
    Alg. 2 and changes them under Alg. 1."""
    cfg, w, model = tiny
    toks = synth.make_tokens(8, 7, cfg["vocab"])
    w2 = dict(w)
    w2["layers"] = [dict(lw) for lw in w["layers"]]
    w2["layers"][1]["wd"] = w["layers"][1]["wd"] * np.float32(1.5)       # MLP of layer 1
    model2 = oracle.Model(cfg, w2, max_ctx=64)
    bounds = [0, 1, 3, 4]                                                  # layers 1, 2 form a set

    def run(m, fuzzy):
        s = oracle.Sequence(m)
        # identical precise prefix for both models: import it from the unperturbed model
        ref = oracle.Sequence(model)
        ref.calibrate(toks[:6])
        s.K[...] = ref.K; s.V[...] = ref.V; s.set_lens(6, 0)
        tap = s.attn_tap()
        s.fuzzy_step(bounds, toks[6]) if fuzzy else s.sequential_step(toks[6])
        return tap.copy(), s.K[:, :, 6].copy(), s.V[:, :, 6].copy()

    t0, k0, v0 = run(model, True)
    t1, k1, v1 = run(model2, True)
    assert np.array_equal(t0[2], t1[2]) and np.array_equal(k0[2], k1[2]) and np.array_equal(v0[2], v1[2])
    assert not np.array_equal(t0[3], t1[3])        # the next set does see the change
    s0, ks0, _ = run(model, False)
    s1, ks1, _ = run(model2, False)
    assert not np.array_equal(s0[2], s1[2]) and not np.array_equal(ks0[2], ks1[2])


@pytest.mark.parametrize("which", ["tiny", "tiny_qwen"])
def test_calibration_equals_sequential_prefill(oracle, request, which):
    """Calibration yields the precise KV: identical bits to token-by-token sequential decoding,
    for any chunking, and whatever fuzzy steps ran before it (they leave no trace)."""
    cfg, w, model = request.getfixturevalue(which)
    toks = synth.make_tokens(9, 14, cfg["vocab"])
    ref = oracle.Sequence(model)
    ref_logits = np.stack([ref.sequential_step(t) for t in toks])

    whole = oracle.Sequence(model)
    lw = whole.calibrate(toks)
    assert np.array_equal(lw, ref_logits)
    assert np.array_equal(whole.K[:, :, :14], ref.K[:, :, :14]) and np.array_equal(whole.V[:, :, :14], ref.V[:, :, :14])

    bounds = oracle.default_groups(cfg["n_layers"], 2, "packed")
    chunked = oracle.Sequence(model)
    rows = [chunked.calibrate(toks[:5])]
    for t in (3, 7, 11):                      # fuzzy steps on arbitrary tokens, all dropped below
        chunked.fuzzy_step(bounds, t)
    assert (chunked.precise, chunked.fuzzy) == (5, 3)
    rows.append(chunked.calibrate(toks[5:6]))
    chunked.fuzzy_step(bounds, 1)
    rows.append(chunked.calibrate(toks[6:14]))
    assert (chunked.precise, chunked.fuzzy) == (14, 0)
    assert np.array_equal(np.concatenate(rows), ref_logits)
    assert np.array_equal(chunked.K[:, :, :14], ref.K[:, :, :14]) and np.array_equal(chunked.V[:, :, :14], ref.V[:, :, :14])
    last = oracle.Sequence(model)
    assert np.array_equal(last.calibrate(toks, all_rows=False), ref_logits[-1])


def test_stale_fuzzy_slots_are_never_read(oracle, tiny):
    """Discarding is a length reset: poisoning every slot at or beyond the precise length
    with NaN changes nothing afterwards."""
    cfg, w, model = tiny
    toks = synth.make_tokens(10, 12, cfg["vocab"])
    bounds = [0, 1, 3, 4]
    a = oracle.Sequence(model)
    a.calibrate(toks[:6])
    for t in toks[6:10]:
        a.fuzzy_step(bounds, t)
    b = a.clone()
    b.K[:, :, 6:] = np.nan; b.V[:, :, 6:] = np.nan
    la, lb = a.calibrate(toks[6:8]), b.calibrate(toks[6:8])
    assert np.array_equal(la, lb)
    b.K[:, :, 8:] = np.nan; b.V[:, :, 8:] = np.nan
    assert np.array_equal(a.fuzzy_step(bounds, toks[8]), b.fuzzy_step(bounds, toks[8]))


@pytest.mark.parametrize("bounds", [[0, 1, 2, 3, 4], [0, 1, 3, 4], [0, 2, 4], [0, 4]])
@pytest.mark.parametrize("gamma", [1, 4])
def test_lossless_greedy_loop(oracle, tiny, bounds, gamma):
    """Greedy speculative decoding returns the base model's greedy output token for token, for
    every grouping of the drafter and every speculation length."""
    cfg, w, draft_model = tiny
    base_model = oracle.Model(cfg, synth.make_weights(cfg, seed=11), max_ctx=64)
    prompt = synth.make_tokens(12, 8, cfg["vocab"])
    want = oracle.vanilla_greedy(oracle.Sequence(base_model), prompt, 24)
    got, accepts = oracle.speculative_greedy(oracle.Sequence(draft_model), oracle.Sequence(base_model),
                                             prompt, bounds, gamma, 24)
    assert got == want
    assert all(0 <= m <= gamma for m in accepts)


def test_self_draft_accepts_everything(oracle, tiny):
    """Draft == base and all sets of size one: every drafted token is accepted.  With real
    layer-parallel sets the drafter is only approximate (sanity: it may reject)."""
    cfg, w, model = tiny
    prompt = synth.make_tokens(13, 8, cfg["vocab"])
    _, accepts = oracle.speculative_greedy(oracle.Sequence(model), oracle.Sequence(model), prompt,
                                           np.arange(5), 4, 20)
    assert all(m == 4 for m in accepts)


def test_bf16_mode_is_close_to_fp32_mode(oracle):
    """The bf16 rounding points perturb, not change, the function (a missed widening of the bit
    patterns or a rounding applied to the residual stream would blow this up)."""
    cfg = synth.model_shape("tiny", dtype="bf16")
    wb = synth.make_weights(cfg, seed=14)
    cfg32 = dict(cfg, dtype="fp32")
    w32 = as_f64(wb)
    w32 = {k: (v.astype(np.float32) if k != "layers" else [{a: b.astype(np.float32) for a, b in lw.items()} for lw in v])
           for k, v in w32.items()}
    toks = synth.make_tokens(15, 10, cfg["vocab"])
    sb, s32 = oracle.Sequence(oracle.Model(cfg, wb, 32)), oracle.Sequence(oracle.Model(cfg32, w32, 32))
    lb, l32 = sb.calibrate(toks), s32.calibrate(toks)
    err = rel_l2(lb, l32)
    assert 1e-5 < err < 2e-2
    kb = sb.K[:, :, :10]
    assert np.array_equal(synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(kb)), kb)    # cache holds bf16 values
