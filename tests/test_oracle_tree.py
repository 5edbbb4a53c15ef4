"""Pins of the oracle's draft: the candidate tree against brute-force
enumeration on tiny vocabularies, the paper's counts, and the Medusa special
case.  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import spec_oracle as O
from tests.test_oracle_pins import _tiny_weights

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _paper_counts():
    out = {}
    with open(os.path.join(GOLDEN, "paper_counts.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                out[k.strip()] = int(v)
    return out


def _brute_force_sequences(w, state_row, last_tok, n, V, state_dtype="f32"):
    """Joint log-probability of every one of the V^n token sequences, by chaining
    single-node evaluations along each path (memoised per prefix)."""
    cache = {}

    def dist(prefix):
        if prefix not in cache:
            cache[prefix] = O.logp_along_path(w, state_row, last_tok, prefix, n, state_dtype=state_dtype)[1]
        return cache[prefix]

    joint = {}
    for seq in itertools.product(range(V), repeat=n):
        joint[seq] = [dist(seq[:i])[seq[i]] for i in range(n)]
    return joint, dist


@pytest.mark.parametrize("seed,V,n,top_k", [(0, 5, 3, (5, 5, 5)), (1, 6, 2, (6, 6)), (2, 4, 3, (4, 4, 4))])
def test_full_branching_tree_is_the_cartesian_product(seed, V, n, top_k):
    rng = np.random.default_rng(seed)
    E, D = 12, 10
    w = _tiny_weights(rng, n, E, D, V)
    state = rng.standard_normal((1, E))
    last = np.array([rng.integers(V)])
    L = V ** n
    B = min(L, 17)
    res = O.draft(w, state, last, top_k, B)
    joint, _ = _brute_force_sequences(w, state[0], int(last[0]), n, V)
    # every sequence appears exactly once
    got = {tuple(t) for t in res.leaf_tokens[0].tolist()}
    assert len(got) == L and got == set(joint.keys())
    # leaf score = joint log-probability
    for leaf in range(L):
        seq = tuple(res.leaf_tokens[0, leaf].tolist())
        assert abs(float(res.leaf_scores[0, leaf]) - sum(joint[seq])) < 1e-5
    # probabilities of all leaves sum to one
    assert abs(np.exp(res.leaf_scores[0].astype(np.float64)).sum() - 1.0) < 1e-5
    # kept candidates = global top-B of the enumeration
    ranked = sorted(joint.items(), key=lambda kv: -sum(kv[1]))
    want = [seq for seq, _ in ranked[:B]]
    assert [tuple(t) for t in res.cand_tokens[0].tolist()] == want
    assert np.all(np.diff(res.cand_scores[0]) <= 0)


@pytest.mark.parametrize("seed,top_k", [(3, (3, 2, 2)), (4, (2, 3, 1)), (5, (1, 1, 4))])
def test_partial_branching_tree_equals_conditional_topk_set(seed, top_k):
    rng = np.random.default_rng(seed)
    V, n, E, D = 6, 3, 9, 14
    w = _tiny_weights(rng, n, E, D, V)
    state = rng.standard_normal((1, E))
    last = np.array([2])
    L = int(np.prod(top_k))
    res = O.draft(w, state, last, top_k, L)
    joint, dist = _brute_force_sequences(w, state[0], 2, n, V)
    want = set()
    for seq in joint:
        ok = True
        for i in range(n):
            top = np.argsort(-dist(seq[:i]), kind="stable")[: top_k[i]]
            ok = ok and seq[i] in top
        if ok:
            want.add(seq)
    got = [tuple(t) for t in res.leaf_tokens[0].tolist()]
    assert len(got) == L == len(want) and set(got) == want
    for leaf, seq in enumerate(got):
        assert abs(float(res.leaf_scores[0, leaf]) - sum(joint[seq])) < 1e-5
    # mixed-radix leaf order: leaf index -> ranks; siblings differ in the last token only
    k_last = top_k[-1]
    for leaf in range(0, L, k_last):
        block = res.leaf_tokens[0, leaf:leaf + k_last]
        assert np.all(block[:, :-1] == block[0, :-1])
        assert len(set(block[:, -1].tolist())) == k_last
    # within a sibling block the scores descend (children are sorted by log-prob)
    for leaf in range(0, L, k_last):
        assert np.all(np.diff(res.leaf_scores[0, leaf:leaf + k_last]) <= 0)


def test_leaf_count_and_pruning_as_printed_in_the_paper():
    counts = _paper_counts()
    rng = np.random.default_rng(8)
    V, E, D = 40, 8, 8
    w = _tiny_weights(rng, 3, E, D, V)
    res = O.draft(w, rng.standard_normal((2, E)), np.array([1, 7]), (6, 3, 2), 5)
    assert res.leaf_tokens.shape == (2, counts["tree_leaves_6_3_2"], 3)
    assert res.cand_tokens.shape == (2, 5, 3)
    # candidates are leaves of the tree, most confident first, and cand_leaf points at them
    for q in range(2):
        for c in range(5):
            leaf = res.cand_leaf[q, c]
            assert np.array_equal(res.cand_tokens[q, c], res.leaf_tokens[q, leaf])
            assert res.cand_scores[q, c] == res.leaf_scores[q, leaf]
        assert np.all(np.diff(res.cand_scores[q]) <= 0)
        rest = np.setdiff1d(np.arange(36), res.cand_leaf[q])
        assert res.leaf_scores[q, rest].max() <= res.cand_scores[q, -1]
    with pytest.raises(ValueError):
        O.draft(w, rng.standard_normal((1, E)), np.array([1]), (6, 3, 2), 37)


def test_sequences_are_independent():
    rng = np.random.default_rng(9)
    V, E, D = 30, 10, 12
    w = _tiny_weights(rng, 3, E, D, V)
    state = rng.standard_normal((3, E))
    last = np.array([3, 29, 0])
    full = O.draft(w, state, last, (4, 3, 2), 10)
    for q in range(3):
        one = O.draft(w, state[q:q + 1], last[q:q + 1], (4, 3, 2), 10)
        assert np.array_equal(one.cand_tokens[0], full.cand_tokens[q])
        assert np.array_equal(one.cand_scores[0], full.cand_scores[q])
        assert np.array_equal(one.cand_leaf[0], full.cand_leaf[q])


def test_no_token_conditioning_gives_a_pure_product():
    """With the embedding weight at zero no stage sees the sampled token (the
    Medusa-like case of Sec. 3.1): every node of a depth shares one state, so the
    per-stage top-k sets do not depend on the path."""
    rng = np.random.default_rng(10)
    V, E, D = 25, 10, 12
    w = _tiny_weights(rng, 3, E, D, V)
    res = O.draft(w, rng.standard_normal((1, E)), np.array([5]), (3, 3, 2), 18, w_s=1.0, w_e=0.0)
    for i in range(3):
        assert np.all(res.topk_tok[i] == res.topk_tok[i][0])
        assert np.allclose(res.states[i], res.states[i][0])
    want = set(itertools.product(res.topk_tok[0][0].tolist(), res.topk_tok[1][0].tolist(),
                                 res.topk_tok[2][0].tolist()))
    assert {tuple(t) for t in res.leaf_tokens[0].tolist()} == want
    # and with conditioning on, the sets do depend on the path
    res2 = O.draft(w, rng.standard_normal((1, E)), np.array([5]), (3, 3, 2), 18)
    assert not np.all(res2.topk_tok[2] == res2.topk_tok[2][0])


def test_token_changes_the_draft_and_state_changes_the_draft():
    rng = np.random.default_rng(11)
    V, E, D = 50, 16, 16
    w = _tiny_weights(rng, 3, E, D, V)
    st = rng.standard_normal((1, E))
    a = O.draft(w, st, np.array([1]), (4, 3, 2), 24)
    b = O.draft(w, st, np.array([2]), (4, 3, 2), 24)
    c = O.draft(w, st + 1.0, np.array([1]), (4, 3, 2), 24)
    assert not np.allclose(a.states[0], b.states[0])
    assert not np.allclose(a.states[0], c.states[0])


def test_stage_uses_its_own_weights_and_parent_state():
    """Stage i+1 must project the state of stage i (not the base state) with
    W_{i+1}, and look the token up in Emb_{i+1}: recompute stage 2 by hand."""
    rng = np.random.default_rng(12)
    V, E, D = 20, 7, 9
    w = _tiny_weights(rng, 2, E, D, V)
    st = rng.standard_normal((1, E))
    res = O.draft(w, st, np.array([3]), (3, 2), 6, w_s=0.7, w_e=0.5)
    s1 = res.states[0][0]
    for j in range(3):
        t = res.topk_tok[0][0, j]
        z = 0.7 * (w["proj"][1] @ s1) + 0.5 * w["emb"][1][t]
        mu = z.mean()
        y = (z - mu) / math.sqrt(((z - mu) ** 2).mean() + 1e-5) * w["ln_gamma"][1] + w["ln_beta"][1]
        s2 = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in y])
        assert np.allclose(res.states[1][j], s2, atol=1e-12)
        l = w["head"][1] @ s2
        lp = l - (l.max() + math.log(np.exp(l - l.max()).sum()))
        assert res.topk_tok[1][j, 0] == int(np.argmax(lp))
        assert abs(res.topk_logp[1][j, 0] - lp.max()) < 1e-6


def test_parameter_count_of_the_7b_shape():
    from paper_2404_19124_amd.workloads import WORKLOADS
    counts = _paper_counts()
    p = WORKLOADS["llama7b_b1"].param_count()
    # "800M-1.1B parameters for a 7B-13B base" (Sec. 3.1): the 7B shape sits at the low end
    assert counts["speculator_params_low"] <= p <= counts["speculator_params_high"]
    assert abs(p - 836.8e6) < 0.1e6


def test_tiny_configuration_matches_stored_oracle_result():
    """Regression pin: the stored file was written by tests/golden/make_tiny_golden.py
    from the oracle alone."""
    from tests.golden.make_tiny_golden import compute
    stored = {}
    with open(os.path.join(GOLDEN, "tiny_b1_seed0.txt")) as f:
        for line in f:
            if line.startswith("#") or "=" not in line:
                continue
            k, v = line.split("=")
            stored[k.strip()] = v.split()
    wl, last, d, v = compute()
    assert int(last[0]) == int(stored["last_tok"][0])
    assert d.cand_leaf[0].tolist() == [int(x) for x in stored["cand_leaf"]]
    assert d.cand_tokens[0].reshape(-1).tolist() == [int(x) for x in stored["cand_tokens"]]
    assert np.allclose(d.cand_scores[0], [float(x) for x in stored["cand_scores"]], atol=2e-6)
    assert v.accept_all[0].tolist() == [int(x) for x in stored["accept_all"]]
    assert int(v.best_cand[0]) == int(stored["best_cand"][0])
    assert int(v.accept_len[0]) == int(stored["accept_len"][0])
    assert v.out_tokens[0].tolist() == [int(x) for x in stored["out_tokens"]]
    # invariants the tiny run must show
    assert d.leaf_tokens.shape == (1, 24, 3)
    assert sorted(d.cand_leaf[0].tolist()) == list(range(24))


def test_leaf_numbering_of_a_hand_built_2_3_2_tree():
    """Leaf index = (j1 * 3 + j2) * 2 + j3 with the FIRST stage most significant (Sec. 4.1: the tree is
    branched head by head), checked on tables written out by hand: token ids spell (stage, row, rank),
    so a swapped significance of two stages, or a child row computed with the wrong radix, shows."""
    top_k = (2, 3, 2)
    # tok_i[row][rank] = 100 * stage + 10 * row + rank  (stage 1-based)
    tok = [np.array([[100, 101]], np.int32),
           np.array([[200, 201, 202], [210, 211, 212]], np.int32),
           np.array([[300, 301], [310, 311], [320, 321], [330, 331], [340, 341], [350, 351]], np.int32)]
    # log-probabilities: powers of two, so every leaf's sum is exact in float32 and identifies its path
    lp = [np.array([[-1.0, -2.0]], np.float32),
          np.array([[-0.5, -4.0, -8.0], [-0.25, -16.0, -32.0]], np.float32),
          np.array([[-0.125, -64.0]] * 6, np.float32)]
    lp[2][3] = [-0.0625, -0.03125]          # the children of path (j1=1, j2=0): row 1 * 3 + 0 = 3
    leaf_tokens, leaf_scores = O.expand_tree(tok, lp, top_k, 1)
    assert leaf_tokens.shape == (1, 12, 3)
    # written out by hand: leaf -> (j1, j2, j3) -> tokens
    want = {0: (100, 200, 300), 1: (100, 200, 301), 2: (100, 201, 310), 5: (100, 202, 321),
            6: (101, 210, 330), 7: (101, 210, 331), 8: (101, 211, 340), 11: (101, 212, 351)}
    for leaf, toks in want.items():
        assert tuple(leaf_tokens[0, leaf].tolist()) == toks, leaf
    assert leaf_scores[0, 0] == np.float32(-1.0 - 0.5 - 0.125)
    assert leaf_scores[0, 7] == np.float32(-2.0 - 0.25 - 0.03125)
    assert leaf_scores[0, 6] == np.float32(-2.0 - 0.25 - 0.0625)
    assert leaf_scores[0, 2] == np.float32(-1.0 - 4.0 - 0.125)
    # the three most confident leaves, by hand: leaf 0 (-1.625), leaf 7 (-2.28125), leaf 6 (-2.3125)
    c_tok, c_sc, c_leaf = O.prune(leaf_tokens, leaf_scores, 3)
    assert c_leaf[0].tolist() == [0, 7, 6]
    assert c_tok[0].tolist() == [[100, 200, 300], [101, 210, 331], [101, 210, 330]]
    assert c_sc[0].tolist() == [-1.625, -2.28125, -2.3125]
