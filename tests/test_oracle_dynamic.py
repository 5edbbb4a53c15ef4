"""Pins of the oracle's per-sequence speculation settings (Sec. 4.2: speculation switched off
above a batch size; Sec. 5: candidates per request swapped dynamically).  CPU only."""
import numpy as np
import pytest

from oracle import spec_oracle as O
from tests.test_oracle_pins import _tiny_weights

N, E, D, V = 3, 12, 10, 9


def _inputs(seed, b):
    rng = np.random.default_rng(seed)
    w = _tiny_weights(rng, N, E, D, V)
    return w, rng.standard_normal((b, E)), rng.integers(0, V, b), rng


def test_uniform_settings_equal_the_plain_batched_draft():
    w, state, last, _ = _inputs(0, 4)
    top_k, B = (3, 2, 2), 5
    plain = O.draft(w, state, last, top_k, B)
    dyn = O.draft_dynamic(w, state, last, [top_k] * 4, [B] * 4, B_pad=B)
    assert np.array_equal(dyn["cand_tokens"], plain.cand_tokens)
    assert np.array_equal(dyn["cand_scores"], plain.cand_scores)
    assert np.array_equal(dyn["cand_leaf"], plain.cand_leaf)
    assert dyn["n_cand"].tolist() == [B] * 4


def test_mixed_batch_off_chain_and_trees_with_padding():
    w, state, last, _ = _inputs(1, 5)
    top_k_seq = [(3, 2, 2), (1, 1, 1), (1, 1, 1), (2, 2, 1), (4, 1, 2)]
    B_seq = [6, 1, 0, 4, 3]
    dyn = O.draft_dynamic(w, state, last, top_k_seq, B_seq, B_pad=7)
    assert dyn["cand_tokens"].shape == (5, 7, 3)
    # speculation off: nothing but padding
    assert (dyn["cand_tokens"][2] == -1).all() and (dyn["cand_leaf"][2] == -1).all()
    assert np.isneginf(dyn["cand_scores"][2]).all()
    for q, Bq in enumerate(B_seq):
        assert (dyn["cand_tokens"][q, Bq:] == -1).all() and (dyn["cand_tokens"][q, :Bq] >= 0).all()
        assert np.isneginf(dyn["cand_scores"][q, Bq:]).all()
        assert np.all(np.diff(dyn["cand_scores"][q, :Bq]) <= 0)
    # the k = 1 chain is greedy decoding of the speculator: each token is the arg-max of the
    # distribution that follows the path so far (brute force, one node at a time)
    path = []
    for i in range(N):
        _, lp = O.logp_along_path(w, state[1], int(last[1]), path, N)
        path.append(int(np.argmax(lp)))
    assert dyn["cand_tokens"][1, 0].tolist() == path
    # a sequence does not depend on its neighbours' settings: same result inside another batch
    other = O.draft_dynamic(w, state[[3, 0]], last[[3, 0]], [top_k_seq[3], (1, 2, 1)], [B_seq[3], 2], B_pad=4)
    assert np.array_equal(other["cand_tokens"][0, :4], dyn["cand_tokens"][3, :4])
    assert np.array_equal(other["cand_scores"][0, :4], dyn["cand_scores"][3, :4])
    # the mix weights are the model's (n = 3 stages), not a function of a sequence's tree
    ws, we = O.mix_weights(N)
    forced = O.draft_dynamic(w, state, last, top_k_seq, B_seq, B_pad=7, w_s=ws, w_e=we)
    assert np.array_equal(forced["cand_tokens"], dyn["cand_tokens"])


def test_the_chain_candidate_is_leaf_zero_of_every_wider_tree():
    # the (1, 1, 1) chain follows rank 0 at every stage: it is leaf 0 of any wider tree, with the same score
    w, state, last, _ = _inputs(2, 2)
    dyn = O.draft_dynamic(w, state, last, [(1, 1, 1), (1, 1, 1)], [1, 1], B_pad=1)
    wide = O.draft(w, state, last, (3, 3, 2), 18)
    for q in range(2):
        at = wide.cand_leaf[q].tolist().index(0)
        assert wide.cand_tokens[q, at].tolist() == dyn["cand_tokens"][q, 0].tolist()
        assert wide.cand_scores[q, at] == dyn["cand_scores"][q, 0]


def _brute_verify_row(logits_row_seq, cand_seq, nc, n):
    """Pure-Python verification of one sequence with nc candidates."""
    if nc == 0:
        return 0, 0, [int(max(range(len(logits_row_seq[0][0])), key=lambda v: (logits_row_seq[0][0][v], -v)))]
    best, best_a = 0, -1
    for c in range(nc):
        a = 0
        while a < n:
            row = logits_row_seq[c][a]
            g = max(range(len(row)), key=lambda v: (row[v], -v))
            if g != cand_seq[c][a]:
                break
            a += 1
        if a > best_a:
            best, best_a = c, a
    row = logits_row_seq[best][best_a]
    bonus = max(range(len(row)), key=lambda v: (row[v], -v))
    return best_a, best, [int(t) for t in cand_seq[best][:best_a]] + [int(bonus)]


def test_verify_dynamic_against_brute_force_and_padding_invariance():
    rng = np.random.default_rng(5)
    b, B, n, Vv = 6, 4, 3, 7
    n_cand = np.array([4, 0, 1, 2, 0, 3])
    cand = rng.integers(0, Vv, (b, B, n)).astype(np.int32)
    for q in range(b):
        cand[q, n_cand[q]:] = -1
    logits = rng.standard_normal((b, B, n + 1, Vv))
    # favour acceptance: boost the speculated token at 70 % of the real positions
    for q in range(b):
        for c in range(n_cand[q]):
            for p in range(n):
                if rng.random() < 0.7:
                    logits[q, c, p, cand[q, c, p]] += 4.0
    r = O.verify_dynamic(logits, cand, n_cand)
    for q in range(b):
        a, best, out = _brute_verify_row(logits[q].tolist(), cand[q].tolist(), int(n_cand[q]), n)
        assert r.accept_len[q] == a and r.best_cand[q] == best and r.n_out[q] == a + 1
        assert r.out_tokens[q, :a + 1].tolist() == out and (r.out_tokens[q, a + 1:] == -1).all()
    assert r.accept_len[[1, 4]].tolist() == [0, 0] and r.n_out[[1, 4]].tolist() == [1, 1]
    assert (r.greedy[1, 1:] == -1).all() and (r.greedy[1, 0, 1:] == -1).all() and r.greedy[1, 0, 0] >= 0
    assert r.accept_len.max() >= 1          # the boosts do produce acceptances
    # padding (-1 never equals a greedy token) does not change the outcome of the plain verify, so for
    # sequences with at least one candidate the two agree on everything a caller consumes
    plain = O.verify(logits, cand)
    act = n_cand > 0
    for name in ("accept_len", "best_cand", "out_tokens", "n_out"):
        assert np.array_equal(getattr(plain, name)[act], getattr(r, name)[act]), name
    # all sequences fully speculating: identical to verify()
    full = O.verify_dynamic(logits, np.where(cand < 0, 0, cand), np.full(b, B))
    plain2 = O.verify(logits, np.where(cand < 0, 0, cand))
    for name in ("accept_len", "best_cand", "out_tokens", "n_out", "greedy", "accept_all"):
        assert np.array_equal(getattr(plain2, name), getattr(full, name)), name
