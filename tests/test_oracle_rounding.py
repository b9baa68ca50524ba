"""CPU pins of the oracle's bf16 rounding points.

The paper states no precision, so a bf16 model's roundings are readings; the oracle keeps them in
two switches (activation mode, KV storage) and these tests pin each of them against something other
than the oracle: the library's bfloat16 cast, the error bound of a two-term sum, and the library
decoder in double precision on the same bf16 weights.  The checks of the two-term rounding are one
function that is also run on planted mistakes, which it must reject.
"""
import numpy as np
import pytest

import easyspec_synth as synth
from test_oracle_pins import as_f64, rel_l2


def _samples():
    rng = np.random.default_rng(0)
    edge = np.float32([1 + 2**-8, 1 + 3 * 2**-8, -(1 + 2**-8), 1 + 2**-9, 1 + 2**-16, 1 + 2**-17 + 2**-23,
                       2**-20 * (1 + 2**-8), 0.0, 255.5, 256.5, -3.0, 1.0 + 2**-7 + 2**-15, 7.0e-5, -1.9921875])
    return np.concatenate([rng.standard_normal(3000).astype(np.float32) * 3, edge,
                           rng.standard_normal(300).astype(np.float32) * 1e-6,
                           (rng.standard_normal(300) * 1e4).astype(np.float32)])


def _library_bf16(x64):
    """float64 array -> float32 -> the library's bfloat16 cast (round to nearest even) -> float64."""
    import torch
    return torch.from_numpy(np.asarray(x64, dtype=np.float64)).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()


def check_pair_round(f):
    """Everything that fixes f(x) = bf16(x) + bf16(x - bf16(x)); raises AssertionError where f is something else."""
    xs = _samples()
    x64 = xs.astype(np.float64)
    got = np.array([f(float(x)) for x in xs])
    hi = _library_bf16(x64)
    lo = _library_bf16(x64 - hi)
    # the definition, term by term, by the library cast
    assert np.array_equal(got, hi + lo), "not bf16(x) + bf16(x - bf16(x))"
    # two bf16 terms carry 16 significant bits: the remainder is below 2^-16 |x| (one term leaves up to 2^-9 |x|)
    assert np.all(np.abs(got - x64) <= 2.0**-16 * np.abs(x64)), "error above 2^-16 |x|"
    # exact where one or two bf16 numbers represent x
    assert np.array_equal(np.array([f(float(v)) for v in hi]), hi), "bf16 values must pass unchanged"
    two = hi[:500] * (1.0 + 2.0**-9)                        # hi + hi * 2^-9: two bf16 numbers
    keep = two.astype(np.float32).astype(np.float64) == two
    assert keep.sum() > 300
    assert np.array_equal(np.array([f(float(v)) for v in two[keep]]), two[keep]), "sums of two bf16 numbers must pass unchanged"
    assert f(1.0 + 2.0**-16) == 1.0 + 2.0**-16
    # the second term rounds to nearest, ties to even: x - hi = 2^-9 (1 + 2^-8) lies halfway between two bf16 numbers
    assert f(1.0 + 2.0**-9 * (1 + 2.0**-8)) == 1.0 + 2.0**-9
    assert f(1.0 + 2.0**-9 * (1 + 3 * 2.0**-8)) == 1.0 + 2.0**-9 * (1 + 2.0**-6)
    # odd function
    assert np.array_equal(np.array([f(-float(x)) for x in xs]), -got), "not odd"


def test_pair_round_against_library_cast_and_bound(oracle):
    """eso_bf16_pair_round: hi == the library's bf16 cast, lo == bf16(x - hi), |x - (hi + lo)| <= 2^-16 |x|,
    exact on representable inputs, ties to even, odd."""
    check_pair_round(oracle.bf16_pair_round)
    xs = _samples().astype(np.float64)
    one_term = np.max(np.abs(_library_bf16(xs) - xs) / np.maximum(np.abs(xs), 1e-300))
    assert one_term > 2.0**-10        # the samples do need the second term


def _trunc_bf16(x):
    """float -> bf16 by chopping the low 16 bits (round toward zero)."""
    u = np.float32(x).view(np.uint32) & np.uint32(0xFFFF0000)
    return float(u.view(np.float32))


@pytest.mark.parametrize("mutant", ["drop_lo", "lo_toward_zero", "hi_toward_zero", "lo_from_rounded_difference_of_double"])
def test_pair_round_check_rejects_planted_mistakes(oracle, mutant):
    """The checker above is not vacuous: each wrong two-term rounding fails it."""
    r = oracle.bf16_round

    def drop_lo(x):
        return r(float(np.float32(x)))

    def lo_toward_zero(x):
        hi = r(float(np.float32(x)))
        return hi + _trunc_bf16(float(np.float32(x)) - hi)

    def hi_toward_zero(x):
        hi = _trunc_bf16(x)
        return hi + r(float(np.float32(x)) - hi)

    def lo_from_rounded_difference_of_double(x):      # three terms' worth: lo is not a bf16 number
        hi = r(float(np.float32(x)))
        return hi + float(np.float32(float(np.float32(x)) - hi))

    f = dict(drop_lo=drop_lo, lo_toward_zero=lo_toward_zero, hi_toward_zero=hi_toward_zero,
             lo_from_rounded_difference_of_double=lo_from_rounded_difference_of_double)[mutant]
    with pytest.raises(AssertionError):
        check_pair_round(f)


def _bf16_tiny(shape="tiny"):
    cfg = synth.model_shape(shape, dtype="bf16")
    w = synth.make_weights(cfg, seed=31)
    return cfg, w


@pytest.mark.parametrize("shape", ["tiny", "tiny_qwen"])
def test_activation_rounding_modes_against_library_decoder(oracle, shape):
    """The library decoder in double precision on the bf16 weights knows no rounding point at all.
    With float32 cache entries the plain mode must equal it; the two-term mode must sit at the 2^-16
    level and the one-term mode at the 2^-9 level, two orders of magnitude further.  A pair rounding
    that lost its second term, or a rounding applied to a vector that should stay unrounded (the
    residual stream, the queries), breaks the ordering or the bounds."""
    from hf_ref import build_hf, hf_prefill
    cfg, w = _bf16_tiny(shape)
    hf = build_hf(cfg, as_f64(w))
    toks = synth.make_tokens(32, 12, cfg["vocab"])
    want, _ = hf_prefill(hf, toks)

    def run(act_mode, kv_bf16):
        m = oracle.Model(cfg, w, 32).set_rounding(act_mode, kv_bf16)
        return oracle.Sequence(m).calibrate(toks)

    e_plain = rel_l2(run(oracle.ACT_PLAIN, False), want)
    e_pair = rel_l2(run(oracle.ACT_PAIR, False), want)
    e_single = rel_l2(run(oracle.ACT_SINGLE, False), want)
    assert e_plain < 1e-6                                   # float32 cache storage is all that is left
    assert 1e-7 < e_pair < 1e-4
    assert 3e-4 < e_single < 2e-2
    assert e_single > 30 * e_pair
    # bf16 cache entries alone: a perturbation of the same order as one-term activations, far above the pair's
    e_kv = rel_l2(run(oracle.ACT_PLAIN, True), want)
    assert 1e-4 < e_kv < 2e-2 and e_kv > 10 * e_pair


def test_default_rounding_of_a_bf16_model_is_pair_and_bf16_cache(oracle):
    """What the tight GPU comparisons use: a bf16 model starts in the two-term mode with a bf16 cache;
    a float32 model rounds nothing."""
    cfg, w = _bf16_tiny()
    toks = synth.make_tokens(33, 9, cfg["vocab"])
    dflt = oracle.Sequence(oracle.Model(cfg, w, 32))
    expl = oracle.Sequence(oracle.Model(cfg, w, 32).set_rounding(oracle.ACT_PAIR, True))
    assert np.array_equal(dflt.calibrate(toks), expl.calibrate(toks))
    k = dflt.K[:, :, :9]
    assert np.array_equal(synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(k)), k)          # cache holds bf16 values
    plain = oracle.Sequence(oracle.Model(cfg, w, 32).set_rounding(oracle.ACT_PLAIN, True))
    ld, lp = oracle.Sequence(oracle.Model(cfg, w, 32)).calibrate(toks), plain.calibrate(toks)
    assert 1e-7 < rel_l2(ld, lp) < 2e-3                                                   # a different, nearby function
    with pytest.raises(ValueError):
        oracle.Model(cfg, w, 32).set_rounding(7, True)


def test_rounding_modes_keep_the_structural_pins(oracle):
    """Whatever the rounding mode: sets of one layer reproduce the sequential step bit for bit and
    calibration reproduces token-by-token decoding bit for bit (the modes change numbers, not structure)."""
    cfg, w = _bf16_tiny()
    toks = synth.make_tokens(34, 10, cfg["vocab"])
    singles = np.arange(cfg["n_layers"] + 1)
    for act, kv in ((oracle.ACT_PLAIN, True), (oracle.ACT_SINGLE, True), (oracle.ACT_PAIR, True), (oracle.ACT_PLAIN, False)):
        m = oracle.Model(cfg, w, 32).set_rounding(act, kv)
        a, b, c = oracle.Sequence(m), oracle.Sequence(m), oracle.Sequence(m)
        ref = np.stack([a.sequential_step(t) for t in toks[:7]])
        assert np.array_equal(b.calibrate(toks[:7]), ref)
        assert np.array_equal(a.K[:, :, :7], b.K[:, :, :7])
        c.calibrate(toks[:6])
        assert np.array_equal(c.fuzzy_step(singles, toks[6]), ref[6])
