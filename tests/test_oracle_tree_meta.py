"""Pins of the oracle's token-tree metadata and step hand-over: invariants that
hold for any input, hand-checked small cases and brute-force reconstructions."""
import itertools

import numpy as np

from oracle import spec_oracle as O


def _paths_from_nodes(meta, q, c, n):
    """Follow parent pointers from the candidate's deepest node back to depth 1."""
    toks = []
    j = int(meta["cand_node"][q, c, n - 1])
    while j >= 0:
        toks.append(int(meta["node_tok"][q, j]))
        j = int(meta["node_parent"][q, j])
    return toks[::-1]


def test_hand_case_two_candidates_sharing_one_token():
    cand = np.array([[[7, 3, 5], [7, 4, 5]]], np.int32)          # share the prefix (7)
    m = O.tree_metadata(cand)
    assert m["n_nodes"][0] == 5
    assert m["node_tok"][0, :5].tolist() == [7, 3, 5, 4, 5]      # order of first appearance
    assert m["node_parent"][0, :5].tolist() == [-1, 0, 1, 0, 3]
    assert m["node_depth"][0, :5].tolist() == [1, 2, 3, 2, 3]
    assert m["cand_node"][0].tolist() == [[0, 1, 2], [0, 3, 4]]
    want = np.zeros((6, 6), np.uint8)
    for i, anc in enumerate([[0], [0, 1], [0, 1, 2], [0, 3], [0, 3, 4]]):
        want[i, anc] = 1
    assert np.array_equal(m["mask"][0], want)
    assert (m["node_tok"][0, 5:] == -1).all() and (m["node_depth"][0, 5:] == 0).all()


def test_same_token_at_different_prefixes_is_not_merged():
    cand = np.array([[[1, 9], [2, 9]]], np.int32)                # the two 9s have different parents
    m = O.tree_metadata(cand)
    assert m["n_nodes"][0] == 4 and m["node_parent"][0, :4].tolist() == [-1, 0, -1, 2]


def test_chain_and_duplicates():
    m = O.tree_metadata(np.array([[[4, 4, 4, 4]]], np.int32))    # B = 1: a chain, causal mask
    assert m["n_nodes"][0] == 4 and np.array_equal(m["mask"][0], np.tril(np.ones((4, 4), np.uint8)))
    m = O.tree_metadata(np.array([[[1, 2], [1, 2], [1, 2]]], np.int32))   # identical candidates
    assert m["n_nodes"][0] == 2 and m["cand_node"][0].tolist() == [[0, 1]] * 3


def test_full_tree_counts_and_invariants():
    # every leaf of a (3, 2, 2) tree as a candidate: 3 + 6 + 12 distinct prefixes
    ks = (3, 2, 2)
    rng = np.random.default_rng(0)
    lv = [rng.permutation(50)[:k] for k in ks]
    cand = np.array([[[lv[0][a], lv[1][b] + 100 * a, lv[2][c] + 1000 * b] for a, b, c in
                      itertools.product(range(3), range(2), range(2))]], np.int32)
    m = O.tree_metadata(cand)
    assert m["n_nodes"][0] == 3 + 6 + 12
    _check_invariants(cand, m)


def _check_invariants(cand, m):
    b, B, n = cand.shape
    for q in range(b):
        N = int(m["n_nodes"][q])
        prefixes = {tuple(cand[q, c, :p + 1]) for c in range(B) for p in range(n)}
        assert N == len(prefixes)                                   # brute force: distinct prefixes
        for c in range(B):
            assert _paths_from_nodes(m, q, c, n) == cand[q, c].tolist()
        depth = m["node_depth"][q, :N]
        assert (m["mask"][q, :N, :N].sum(axis=1) == depth).all()    # a node sees itself and its ancestors
        par = m["node_parent"][q, :N]
        assert (par < np.arange(N)).all()                           # parents come first
        assert ((par == -1) == (depth == 1)).all()
        assert (m["mask"][q, N:, :] == 0).all() and (m["mask"][q, :, N:] == 0).all()


def test_random_candidates_with_small_vocabulary():
    rng = np.random.default_rng(3)
    for b, B, n, V in [(3, 8, 3, 3), (2, 16, 4, 2), (1, 5, 7, 2), (4, 1, 5, 10)]:
        cand = rng.integers(0, V, (b, B, n)).astype(np.int32)
        _check_invariants(cand, O.tree_metadata(cand))


def test_advance_picks_state_and_bonus_token():
    rng = np.random.default_rng(1)
    b, B, n, E = 3, 4, 3, 5
    hidden = rng.normal(size=(b, B, n + 1, E))
    best = np.array([2, 0, 3]); acc = np.array([0, 3, 1])
    out = np.array([[11, -1, -1, -1], [5, 6, 7, 8], [9, 10, -1, -1]], np.int32)
    s, t = O.advance(hidden, best, acc, out)
    assert t.tolist() == [11, 8, 10]
    for q in range(b):
        assert np.array_equal(s[q], hidden[q, best[q], acc[q]])
    # consistent with verify: the bonus token is the greedy token at position accept_len
    logits = rng.normal(size=(b, B, n + 1, 20))
    cand = rng.integers(0, 20, (b, B, n)).astype(np.int32)
    v = O.verify(logits, cand)
    _, t2 = O.advance(hidden, v.best_cand, v.accept_len, v.out_tokens)
    for q in range(b):
        assert t2[q] == np.argmax(logits[q, v.best_cand[q], v.accept_len[q]])
