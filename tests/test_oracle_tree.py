"""CPU pins of the oracle's token-tree fuzzy step (paper Sec. 3.1 last paragraph, App. C).

A token tree shares the KV entries of common prefixes and gives every node the attention row
of its own root-to-node sequence.  So each path of the tree must reproduce, bit for bit, what
chain drafting of that path alone produces (logits, hidden states and the k, v stored for the
node), whatever else is in the tree; chain drafting itself is pinned in test_oracle_pins.py."""
import numpy as np
import pytest

import easyspec_synth as synth

BOUNDS = [[0, 1, 3, 4], [0, 4], [0, 1, 2, 3, 4]]


def setup(oracle, seed=50, prompt_len=9, **over):
    cfg = synth.model_shape("tiny", **over)
    w = synth.make_weights(cfg, seed)
    seq = oracle.Sequence(oracle.Model(cfg, w, 128))
    prompt = synth.make_tokens(seed + 1, prompt_len, cfg["vocab"])
    seq.calibrate(prompt)
    return cfg, seq


@pytest.mark.parametrize("bounds", BOUNDS)
def test_chain_shaped_tree_is_chain_drafting(oracle, bounds):
    cfg, seq = setup(oracle)
    ref = seq.clone()
    toks = synth.make_tokens(3, 5, cfg["vocab"])
    for j, t in enumerate(toks):
        lt, ht = seq.fuzzy_tree_step(bounds, [t], [j - 1], want_hidden=True)
        lc, hc = ref.fuzzy_step(bounds, t, want_hidden=True)
        assert np.array_equal(lt[0], lc) and np.array_equal(ht[0], hc)
    assert (seq.precise, seq.fuzzy) == (ref.precise, ref.fuzzy)
    n = seq.precise + seq.fuzzy
    assert np.array_equal(seq.K[:, :, :n], ref.K[:, :, :n]) and np.array_equal(seq.V[:, :, :n], ref.V[:, :, :n])


@pytest.mark.parametrize("bounds", BOUNDS)
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_every_path_of_a_tree_equals_its_chain(oracle, bounds, dtype):
    """Tree (node: parent):  level 1: 0:-1 1:-1 2:-1 | level 2: 3:0 4:0 5:2 | level 3: 6:4 7:5 8:5 | level 4: 9:8."""
    cfg, seq = setup(oracle, dtype=dtype)
    base = seq.clone()
    P = seq.precise
    levels = [([-1, -1, -1]), ([0, 0, 2]), ([4, 5, 5]), ([8])]
    toks = synth.make_tokens(4, 10, cfg["vocab"])
    parent, logits, hidden = {}, {}, {}
    node = 0
    for parents in levels:
        t = toks[node:node + len(parents)]
        lg, hd = seq.fuzzy_tree_step(bounds, t, parents, want_hidden=True)
        for j, p in enumerate(parents):
            parent[node], logits[node], hidden[node] = p, lg[j], hd[j]
            node += 1
    assert (seq.precise, seq.fuzzy) == (P, 10)
    for leaf in (1, 3, 6, 7, 9):
        path = []
        t = leaf
        while t >= 0:
            path.append(t)
            t = parent[t]
        path.reverse()
        ref = base.clone()
        for depth, t in enumerate(path):
            lc, hc = ref.fuzzy_step(bounds, toks[t], want_hidden=True)
            assert np.array_equal(lc, logits[t]), (leaf, t)
            assert np.array_equal(hc, hidden[t])
            # the node's k, v (tree slot P + t) are the chain's at slot P + depth
            assert np.array_equal(seq.K[:, :, P + t], ref.K[:, :, P + depth])
            assert np.array_equal(seq.V[:, :, P + t], ref.V[:, :, P + depth])


def test_siblings_do_not_see_each_other_but_children_see_parents(oracle):
    cfg, seq = setup(oracle)
    other = seq.clone()
    b = BOUNDS[0]
    a = seq.fuzzy_tree_step(b, [5, 6], [-1, -1])
    c = other.fuzzy_tree_step(b, [5, 7], [-1, -1])          # different sibling
    assert np.array_equal(a[0], c[0]) and not np.array_equal(a[1], c[1])
    a2 = seq.fuzzy_tree_step(b, [9, 9], [0, 1])
    c2 = other.fuzzy_tree_step(b, [9, 9], [0, 1])
    assert np.array_equal(a2[0], c2[0])                      # child of the common node: same
    assert not np.array_equal(a2[1], c2[1])                  # child of the differing node: differs
    assert not np.array_equal(a2[0], a2[1])                  # same token, different parents


def test_calibration_after_a_tree_leaves_no_trace(oracle):
    cfg, seq = setup(oracle)
    clean = seq.clone()
    b = BOUNDS[0]
    seq.fuzzy_tree_step(b, [1, 2, 3, 4], [-1, -1, -1, -1])
    seq.fuzzy_tree_step(b, [5, 6, 7], [0, 0, 3])
    toks = [2, 6, 11]
    assert np.array_equal(seq.calibrate(toks), clean.calibrate(toks))
    n = seq.precise
    assert np.array_equal(seq.K[:, :, :n], clean.K[:, :, :n])
    # and a new tree can start afterwards
    assert np.array_equal(seq.fuzzy_tree_step(b, [4], [-1]), clean.fuzzy_tree_step(b, [4], [-1]))


def test_tree_step_rejects_bad_input(oracle):
    cfg, seq = setup(oracle)
    b = BOUNDS[0]
    with pytest.raises(RuntimeError):
        seq.fuzzy_tree_step(b, [1], [0])                     # parent that does not exist yet
    seq.fuzzy_tree_step(b, [1, 2], [-1, -1])
    with pytest.raises(RuntimeError):
        seq.fuzzy_tree_step(b, [1, 2], [0, 2])               # parent inside the same level
    with pytest.raises(RuntimeError):
        seq.fuzzy_step(b, 3)                                 # chain step into a tree
    chain = setup(oracle)[1]
    chain.fuzzy_step(b, 3)
    with pytest.raises(RuntimeError):
        chain.fuzzy_tree_step(b, [1], [-1])                  # tree step after chain-drafted slots
    full = setup(oracle)[1]
    for lvl in range(4):
        full.fuzzy_tree_step(b, list(range(12)), [-1] * 12 if lvl == 0 else [0] * 12)
    full.fuzzy_tree_step(b, list(range(12)), [0] * 12)       # 60 nodes
    with pytest.raises(RuntimeError):
        full.fuzzy_tree_step(b, list(range(5)), [0] * 5)     # 65 > 64 nodes
