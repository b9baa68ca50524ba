"""GPU parity of acceptance by speculative sampling (paper Alg. 3, Sec. 2.1): the device entry
point against the CPU oracle on the same logits, drafted tokens and uniform random numbers.
accept_len and bonus are integers and must be equal; both sides compute in double precision,
and a case is set aside only if the oracle reports that one of its decisions lies within 1e-9
(relative) of its threshold, where the order of a sum could move it (counted, asserted rare)."""
import numpy as np
import pytest

import easyspec_synth as synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def es():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device; none is visible")
    import paper_2502_02493_amd as es
    return es


def make_case(seed, batch, gamma, V, T, noise):
    """Target logits N(0, 2); draft logits = target + N(0, noise) so that acceptance ratios spread over
    (0, 1]; drafted tokens drawn from the draft distribution."""
    tl = synth.make_logits(seed, batch * (gamma + 1), V).reshape(batch, gamma + 1, V)
    dl = (tl[:, :gamma] + synth.make_logits(seed + 1, batch * gamma, V, std=noise).reshape(batch, gamma, V)).astype(np.float32)
    ru = synth.make_uniforms(seed + 2, batch * (2 * gamma + 1))
    r = ru[:batch * gamma].reshape(batch, gamma).copy()
    u = ru[batch * gamma:batch * (gamma + 1)].copy()
    pick = ru[batch * (gamma + 1):].reshape(batch, gamma)
    z = dl.astype(np.float64) / T
    pd = np.exp(z - z.max(axis=-1, keepdims=True))
    cum = np.cumsum(pd, axis=-1)
    draft = np.zeros((batch, gamma), np.int32)
    for b in range(batch):
        for i in range(gamma):
            draft[b, i] = min(V - 1, int(np.searchsorted(cum[b, i], pick[b, i] * cum[b, i, -1], side="right")))
    return draft, dl, tl, r, u


def run_gpu(es, draft, dl, tl, r, u, T):
    import torch
    batch, gamma = draft.shape
    V = tl.shape[-1]
    dev = torch.device("cuda:0")
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    d_draft, d_dl, d_tl, d_r, d_u = t(draft), t(dl), t(tl), t(r), t(u)
    acc = torch.full((batch,), -7, dtype=torch.int32, device=dev)
    bon = torch.full((batch,), -7, dtype=torch.int32, device=dev)
    ws = torch.empty(es.easyspec_accept_workspace_bytes(batch, gamma, V) // 8, dtype=torch.float64, device=dev)
    es.easyspec_accept(d_draft if gamma else None, d_dl if gamma else None, d_tl, d_r if gamma else None, d_u, batch, gamma, V, T,
                       acc, bon, ws, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return acc.cpu().numpy(), bon.cpu().numpy()


@pytest.mark.parametrize("batch,gamma,V,T,noise", [
    (1, 1, 7, 1.0, 1.0),            # smaller than one wave
    (5, 5, 1000, 0.8, 0.7),         # the paper's temperature and speculation length
    (3, 8, 1031, 1.3, 1.5),         # vocabulary not a multiple of anything; long speculation
    (2, 0, 513, 0.8, 1.0),          # no drafted token: plain sampling from p_0
    (16, 5, 4099, 0.8, 0.3),        # close distributions: long accepted prefixes
    (4, 5, 128256, 0.8, 0.7),       # full-size vocabulary of the 8B shape
])
def test_accept_parity(oracle, es, batch, gamma, V, T, noise):
    draft, dl, tl, r, u = make_case(1000 + V, batch, gamma, V, T, noise)
    acc, bon = run_gpu(es, draft, dl, tl, r, u, T)
    checked = skipped = 0
    lens = []
    for b in range(batch):
        m, bonus, margin = oracle.accept(draft[b], dl[b], tl[b], r[b], u[b], T, with_margin=True)
        if margin > 1e-9:
            assert (int(acc[b]), int(bon[b])) == (m, bonus), (b, margin)
            checked += 1
        else:
            skipped += 1
        lens.append(m)
    assert skipped <= max(1, batch // 8), (checked, skipped)
    if batch >= 5 and gamma >= 5:
        assert len(set(lens)) > 1, "inputs should exercise several acceptance lengths"


def test_accept_distribution_on_device(oracle, es):
    """4000 independent sequences with the same pair of distributions in one call: the first
    output token (drafted token if accepted, else the bonus token) follows the target
    distribution (chi-square, 5 degrees of freedom, 0.1 % level)."""
    V, n = 6, 4000
    rng = np.random.default_rng(5)
    p = rng.random(V) + 0.05
    p /= p.sum()
    pd = rng.random(V) + 0.05
    pd /= pd.sum()
    tl = np.broadcast_to(np.stack([np.log(p), np.log(p[::-1])]).astype(np.float32), (n, 2, V)).copy()
    dl = np.broadcast_to(np.log(pd).astype(np.float32), (n, 1, V)).copy()
    ru = synth.make_uniforms(77, 3 * n).reshape(3, n)
    draft = np.minimum(V - 1, np.searchsorted(np.cumsum(pd), ru[0], side="right")).astype(np.int32).reshape(n, 1)
    acc, bon = run_gpu(es, draft, dl, tl, ru[1].reshape(n, 1).copy(), ru[2].copy(), 1.0)
    out = np.where(acc == 1, draft[:, 0], bon)
    counts = np.bincount(out, minlength=V)
    chi2 = float(np.sum((counts - n * p) ** 2 / (n * p)))
    assert chi2 < 20.5, chi2
    # and every sequence equals the oracle's result
    for b in range(0, n, 97):
        assert (int(acc[b]), int(bon[b])) == oracle.accept(draft[b], dl[b], tl[b], [ru[1, b]], ru[2, b], 1.0)


def test_accept_flags_a_bad_token(es):
    draft, dl, tl, r, u = make_case(3, 2, 3, 50, 1.0, 1.0)
    draft[1, 0] = 50          # positions after the first rejection are never looked at, so plant it first
    acc, bon = run_gpu(es, draft, dl, tl, r, u, 1.0)
    assert acc[1] == -1 and bon[1] == -1 and acc[0] >= 0 and 0 <= bon[0] < 50
