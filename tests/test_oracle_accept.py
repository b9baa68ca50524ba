"""CPU pins of the oracle's acceptance by speculative sampling (paper Alg. 3, Sec. 2.1).

The algorithm is an exact sampler of the target distribution whatever the draft distribution
is (the paper's closing remark of App. A).  That property, checked by exact integration over the
random inputs on tiny vocabularies, fixes every step at once: a wrong acceptance ratio, a
residual with the wrong sign or without normalisation, or the distributions of the wrong
position all change the output distribution.  Hand-computed cases and the reductions to greedy
acceptance and to plain inverse-CDF sampling pin the rest."""
import ctypes as C

import numpy as np
import pytest

import easyspec_synth as synth


def probs_to_logits(p):
    return np.log(np.asarray(p, dtype=np.float64)).astype(np.float32)


class FastAccept:
    """The oracle entry point with preallocated arguments (hundreds of thousands of calls)."""

    def __init__(self, oracle, gamma, V, T=1.0):
        self.lib, self.gamma, self.V, self.T = oracle.lib(), gamma, V, T
        self.draft = np.zeros(gamma, np.int32)
        self.dl = np.zeros((gamma, V), np.float32)
        self.tl = np.zeros((gamma + 1, V), np.float32)
        self.r = np.zeros(gamma, np.float32)
        self.m, self.b = C.c_int32(), C.c_int32()
        fp, ip = C.POINTER(C.c_float), C.POINTER(C.c_int32)
        self.args = (self.draft.ctypes.data_as(ip), self.dl.ctypes.data_as(fp), self.tl.ctypes.data_as(fp),
                     self.r.ctypes.data_as(fp))

    def __call__(self, u):
        rc = self.lib.eso_accept(*self.args, C.c_float(u), self.gamma, self.V, C.c_double(self.T), C.byref(self.m),
                                 C.byref(self.b), None)
        assert rc == 0
        return self.m.value, self.b.value


def random_dist(rng, V, zeros=0):
    p = rng.random(V) + 0.05
    if zeros:
        p[rng.choice(V, zeros, replace=False)] = 1e-30      # practically impossible tokens
    return p / p.sum()


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_output_distribution_equals_target_gamma1(oracle, seed):
    """One drafted token: P(first output token = v) = p(v), by midpoint integration over r and u."""
    rng = np.random.default_rng(seed)
    V, N = 4, 240
    p, pd = random_dist(rng, V), random_dist(rng, V)
    f = FastAccept(oracle, 1, V)
    f.dl[0] = probs_to_logits(pd)
    f.tl[0] = probs_to_logits(p)
    f.tl[1] = probs_to_logits(random_dist(rng, V))
    grid = (np.arange(N) + 0.5) / N
    out = np.zeros(V)
    for x in range(V):
        f.draft[0] = x
        for r in grid:
            f.r[0] = r
            # the bonus draw matters only after a rejection
            m, b = f(0.5)
            if m == 1:
                out[x] += pd[x] / N
            else:
                for u in grid:
                    m, b = f(u)
                    out[b] += pd[x] / (N * N)
    assert abs(out.sum() - 1) < 1e-9
    assert np.max(np.abs(out - p)) < 2.5 / N, (out, p)


def test_output_distribution_equals_target_gamma2(oracle):
    """Two drafted tokens with distributions that depend on the first token: the first output
    token follows p_1, the second (when the first was accepted) follows p_2(. | first), and the
    token after two acceptances follows p_3."""
    rng = np.random.default_rng(7)
    V, N = 3, 24
    pd1, p1 = random_dist(rng, V), random_dist(rng, V)
    pd2 = [random_dist(rng, V) for _ in range(V)]
    p2 = [random_dist(rng, V) for _ in range(V)]
    p3 = random_dist(rng, V)
    f = FastAccept(oracle, 2, V)
    grid = (np.arange(N) + 0.5) / N
    first = np.zeros(V)
    second = np.zeros((V, V))
    third = np.zeros(V)
    mass_first_ok = np.zeros(V)
    mass_both_ok = 0.0
    for x1 in range(V):
        for x2 in range(V):
            w = pd1[x1] * pd2[x1][x2] / N ** 3
            f.draft[:] = (x1, x2)
            f.dl[0], f.dl[1] = probs_to_logits(pd1), probs_to_logits(pd2[x1])
            f.tl[0], f.tl[1], f.tl[2] = probs_to_logits(p1), probs_to_logits(p2[x1]), probs_to_logits(p3)
            for r1 in grid:
                for r2 in grid:
                    f.r[:] = (r1, r2)
                    for u in grid:
                        m, b = f(u)
                        if m == 0:
                            first[b] += w
                        else:
                            first[x1] += w
                            mass_first_ok[x1] += w
                            if m == 1:
                                second[x1, b] += w
                            else:
                                second[x1, x2] += w
                                third[b] += w
                                mass_both_ok += w
    tol = 4.0 / N
    assert np.max(np.abs(first - p1)) < tol
    for a in range(V):
        assert np.max(np.abs(second[a] / mass_first_ok[a] - p2[a])) < tol
    assert np.max(np.abs(third / mass_both_ok - p3)) < tol


def test_hand_computed_case(oracle):
    """p = (3/4, 1/4), p' = (1/4, 3/4), drafted token 1: acceptance ratio 1/3; after a rejection the
    residual max(0, p - p') = (1/2, 0) puts all mass on token 0.  Drafted token 0: ratio 3 > 1,
    always accepted, and the bonus then comes from the next position's target distribution."""
    tl = np.stack([probs_to_logits([0.75, 0.25]), probs_to_logits([0.1, 0.9])])
    dl = probs_to_logits([0.25, 0.75])[None]
    assert oracle.accept([1], dl, tl, [0.33], 0.99, 1.0) == (1, 1)      # accepted; bonus from (0.1, 0.9), u = 0.99
    assert oracle.accept([1], dl, tl, [0.33], 0.05, 1.0) == (1, 0)
    assert oracle.accept([1], dl, tl, [0.34], 0.99, 1.0) == (0, 0)      # rejected; residual is one-hot on token 0
    assert oracle.accept([1], dl, tl, [0.34], 0.0, 1.0) == (0, 0)
    assert oracle.accept([0], dl, tl, [0.999], 0.5, 1.0) == (1, 1)
    # three tokens, rejection at the second position: the residual of THAT position is used
    tl3 = np.stack([probs_to_logits([0.5, 0.5]), probs_to_logits([0.2, 0.8]), probs_to_logits([0.5, 0.5])])
    dl3 = np.stack([probs_to_logits([0.5, 0.5]), probs_to_logits([0.9, 0.1])])
    # position 0: ratio 1 -> accepted for any r < 1; position 1, token 0: ratio 2/9
    assert oracle.accept([1, 0], dl3, tl3, [0.9, 0.3], 0.5, 1.0) == (1, 1)   # residual (0, 0.7) -> token 1
    assert oracle.accept([1, 0], dl3, tl3, [0.9, 0.2], 0.4, 1.0) == (2, 0)   # all accepted, bonus from (0.5, 0.5)
    assert oracle.accept([1, 0], dl3, tl3, [0.9, 0.2], 0.6, 1.0) == (2, 1)


def test_identical_distributions_accept_everything_and_bonus_is_inverse_cdf(oracle):
    rng = np.random.default_rng(11)
    V, gamma = 50, 4
    tl = rng.normal(size=(gamma + 1, V)).astype(np.float32) * 2
    draft = rng.integers(0, V, gamma)
    for T in (0.5, 1.0, 1.7):
        z = tl[gamma].astype(np.float64) / T
        p = np.exp(z - z.max())
        cum = np.cumsum(p)
        for u in rng.random(20).astype(np.float32):
            m, b, mg = oracle.accept(draft, tl[:gamma], tl, rng.random(gamma) * 0.999, u, T, with_margin=True)
            assert m == gamma
            thr = float(u) * cum[-1]
            want = int(np.searchsorted(cum, thr, side="right"))
            gap = min(cum[want] - thr, thr - cum[want - 1] if want else np.inf) / cum[-1]
            if gap > 1e-9:      # this test's own distance to the neighbouring outcomes
                assert b == want
                assert abs(mg - gap) < 1e-9 or mg < gap      # the reported margin is no larger than the true one


def test_zero_r_accepts_everything(oracle):
    rng = np.random.default_rng(12)
    V, gamma = 17, 5
    tl = rng.normal(size=(gamma + 1, V)).astype(np.float32) * 3
    dl = rng.normal(size=(gamma, V)).astype(np.float32) * 3
    m, _ = oracle.accept(rng.integers(0, V, gamma), dl, tl, np.zeros(gamma), 0.3, 0.8)
    assert m == gamma


def test_sharp_distributions_reduce_to_greedy_accept(oracle):
    """Temperature -> 0 turns both distributions one-hot; a drafted token that is the draft's own
    argmax is then accepted exactly when it is the target's argmax, and the bonus token is the
    target's argmax at the first rejected (or the extra) position: greedy acceptance."""
    rng = np.random.default_rng(13)
    V, gamma = 9, 6
    for _ in range(50):
        tl = rng.normal(size=(gamma + 1, V)).astype(np.float32)
        dl = rng.normal(size=(gamma, V)).astype(np.float32)
        # make the draft agree with the target on a random prefix
        k = rng.integers(0, gamma + 1)
        dl[:k] = tl[:k]
        draft = dl.argmax(axis=1)
        target = tl.argmax(axis=1)
        want = oracle.greedy_accept(draft, target)
        got = oracle.accept(draft, dl, tl, rng.random(gamma) * 0.98 + 0.01, rng.random(), 1e-3)
        assert got == want


def test_temperature_is_a_scaling_of_the_logits(oracle):
    rng = np.random.default_rng(14)
    V, gamma = 33, 3
    tl = rng.normal(size=(gamma + 1, V)).astype(np.float32)
    dl = rng.normal(size=(gamma, V)).astype(np.float32)
    draft = rng.integers(0, V, gamma)
    for _ in range(30):
        r, u = rng.random(gamma), rng.random()
        assert oracle.accept(draft, dl, tl, r, u, 2.0) == oracle.accept(draft, dl / 2, tl / 2, r, u, 1.0)


def test_chi_square_with_generated_uniforms(oracle):
    """Distributional check with the seeded generator's uniforms (what the GPU tests feed to both sides)."""
    V, n = 6, 6000
    rng = np.random.default_rng(15)
    p, pd = random_dist(rng, V), random_dist(rng, V)
    tl = np.stack([probs_to_logits(p), probs_to_logits(random_dist(rng, V))])
    dl = probs_to_logits(pd)[None]
    ru = synth.make_uniforms(21, n * 3).reshape(n, 3)
    counts = np.zeros(V)
    for i in range(n):
        x = int(np.searchsorted(np.cumsum(pd), ru[i, 0] * 1.0, side="right").clip(0, V - 1))
        m, b = oracle.accept([x], dl, tl, [ru[i, 1]], ru[i, 2], 1.0)
        counts[x if m == 1 else b] += 1
    chi2 = float(np.sum((counts - n * p) ** 2 / (n * p)))
    assert chi2 < 20.5, chi2          # 5 degrees of freedom: P(chi2 > 20.5) = 0.001


def test_bad_arguments(oracle):
    with pytest.raises(ValueError):
        oracle.accept([5], np.zeros((1, 3), np.float32), np.zeros((2, 3), np.float32), [0.5], 0.5, 1.0)   # token out of range
    with pytest.raises(ValueError):
        oracle.accept([0], np.zeros((1, 3), np.float32), np.zeros((2, 3), np.float32), [0.5], 0.5, 0.0)   # temperature 0
