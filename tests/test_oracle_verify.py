"""Pins of the oracle's verify step: brute-force longest-prefix matching, the
bounds the paper states (0..n accepted, always one bonus token), tie rules and
the shape of the flattened verification batch.  CPU only."""
import numpy as np
import pytest

from oracle import spec_oracle as O
from tests.test_oracle_tree import _paper_counts


def _brute_verify(logits, cand):
    """Independent pure-Python restatement on lists: longest matching prefix."""
    b, B, n1, V = logits.shape
    n = n1 - 1
    out = []
    for q in range(b):
        best, best_len = 0, -1
        for c in range(B):
            g = [max(range(V), key=lambda v: (logits[q, c, p, v], -v)) for p in range(n1)]
            m = 0
            for p in range(n):
                if all(g[i] == cand[q, c, i] for i in range(p + 1)):
                    m = p + 1
            if m > best_len:
                best, best_len, best_g = c, m, g
        toks = [int(cand[q, best, i]) for i in range(best_len)] + [best_g[best_len]]
        out.append((best, best_len, toks))
    return out


def _random_case(rng, b, B, n, V, p_match):
    logits = rng.standard_normal((b, B, n + 1, V)).astype(np.float32)
    cand = rng.integers(0, V, (b, B, n)).astype(np.int32)
    hit = rng.random((b, B, n)) < p_match
    for q in range(b):
        for c in range(B):
            for p in range(n):
                if hit[q, c, p]:
                    logits[q, c, p, cand[q, c, p]] += 20.0
    return logits, cand


@pytest.mark.parametrize("seed,b,B,n,V,p", [(0, 3, 5, 3, 17, 0.7), (1, 2, 8, 4, 9, 0.8), (2, 4, 1, 7, 12, 0.9),
                                            (3, 1, 6, 1, 5, 0.5), (4, 5, 4, 3, 33, 0.0)])
def test_verify_equals_brute_force(seed, b, B, n, V, p):
    rng = np.random.default_rng(seed)
    logits, cand = _random_case(rng, b, B, n, V, p)
    res = O.verify(logits, cand)
    want = _brute_verify(logits, cand)
    for q in range(b):
        best, a, toks = want[q]
        assert res.best_cand[q] == best
        assert res.accept_len[q] == a
        assert res.n_out[q] == a + 1
        assert res.out_tokens[q, :a + 1].tolist() == toks
        assert np.all(res.out_tokens[q, a + 1:] == -1)
    # bounds stated by the paper: at most n accepted, always one bonus token
    assert res.accept_len.min() >= 0 and res.accept_len.max() <= n
    assert res.n_out.min() >= 1 and res.n_out.max() <= n + 1


def test_all_matching_gives_n_plus_one_tokens_and_uses_position_n():
    counts = _paper_counts()
    rng = np.random.default_rng(5)
    b, B, n, V = 2, 3, 3, 50
    logits, cand = _random_case(rng, b, B, n, V, 1.0)
    logits[:, :, n, 7] += 30.0            # bonus token comes from the position after the last speculated one
    res = O.verify(logits, cand)
    assert np.all(res.accept_len == n)
    assert np.all(res.n_out == counts["max_tokens_per_step_n3"])
    assert np.all(res.best_cand == 0)      # all tie at n: first candidate
    assert np.all(res.out_tokens[:, :n] == cand[:, 0, :])
    assert np.all(res.out_tokens[:, n] == 7)


def test_nothing_matching_gives_exactly_the_base_token():
    rng = np.random.default_rng(6)
    b, B, n, V = 3, 4, 3, 1000
    logits = rng.standard_normal((b, B, n + 1, V)).astype(np.float32)
    greedy0 = logits[:, :, 0, :].argmax(-1)
    cand = ((greedy0[:, :, None] + 1 + np.arange(n)) % V).astype(np.int32)   # never the greedy token at position 0
    res = O.verify(logits, cand)
    assert np.all(res.accept_len == 0) and np.all(res.n_out == 1) and np.all(res.best_cand == 0)
    assert np.array_equal(res.out_tokens[:, 0], greedy0[:, 0])
    assert np.all(res.out_tokens[:, 1:] == -1)


def test_a_match_after_a_mismatch_does_not_count():
    V, n = 10, 3
    logits = np.zeros((1, 1, n + 1, V), np.float32)
    cand = np.array([[[1, 2, 3]]], np.int32)
    logits[0, 0, 0, 1] = 5      # match
    logits[0, 0, 1, 9] = 5      # mismatch (speculated 2)
    logits[0, 0, 2, 3] = 5      # would match, but comes after a mismatch
    res = O.verify(logits, cand)
    assert res.accept_len[0] == 1
    assert res.out_tokens[0].tolist() == [1, 9, -1, -1]


def test_ties_in_logits_and_between_candidates():
    V, n = 8, 2
    logits = np.zeros((1, 3, n + 1, V), np.float32)        # all-equal rows: greedy token is index 0
    cand = np.array([[[1, 0], [0, 1], [0, 0]]], np.int32)
    res = O.verify(logits, cand)
    assert np.all(res.greedy == 0)
    assert res.accept_all[0].tolist() == [0, 1, 2]
    assert res.best_cand[0] == 2 and res.accept_len[0] == 2
    logits[0, :, :, 5] = 1.0
    logits[0, :, :, 3] = 1.0                                # two maxima: the smaller index wins
    res = O.verify(logits, np.array([[[3, 3], [3, 5], [5, 3]]], np.int32))
    assert np.all(res.greedy == 3)
    assert res.accept_all[0].tolist() == [2, 1, 0]
    # equal accepted lengths: the first candidate is kept
    res = O.verify(logits, np.array([[[3, 5], [3, 0], [3, 1]]], np.int32))
    assert res.best_cand[0] == 0 and res.accept_len[0] == 1
    assert res.out_tokens[0].tolist() == [3, 3, -1]


def test_bf16_valued_logits_tie_to_the_smallest_index():
    import torch
    g = torch.Generator().manual_seed(0)
    x = torch.randn(64, 20000, generator=g).to(torch.bfloat16)
    xf = x.float().numpy()
    res = O.verify(xf.reshape(1, 16, 4, 20000), np.zeros((1, 16, 3), np.int32))
    ties = 0
    for r in range(64):
        row = xf[r]
        m = row.max()
        first = int(np.flatnonzero(row == m)[0])
        ties += int((row == m).sum() > 1)
        assert res.greedy.reshape(-1)[r] == first
    assert ties > 0          # the case really occurs with bf16 logits


def test_flattened_batch_shape_as_in_the_paper():
    counts = _paper_counts()
    b, k, n = 4, 32, 3
    assert b * k * (n + 1) == counts["verify_tokens_b4_k32"]
    assert n + 1 == counts["tokens_per_candidate_n3"] and 7 + 1 == counts["tokens_per_candidate_n7"]
    rng = np.random.default_rng(7)
    logits = rng.standard_normal((b, k, n + 1, 6)).astype(np.float32)
    res = O.verify(logits, rng.integers(0, 6, (b, k, n)).astype(np.int32))
    assert res.greedy.size == counts["verify_tokens_b4_k32"]
