"""The comparator of the GPU parity tests, checked on the CPU: fed with the oracle's own
tables it reports an exact match; a planted mistake (in a copy of the oracle's tables, never
on a device) is rejected unless it is a near-tie inside the strict 1e-3 band."""
import numpy as np
import pytest

from oracle import spec_oracle as O
from tests import parity
from tests.test_oracle_pins import _tiny_weights

N, TOP_K, BATCH, KEEP, E, D, V = 3, (3, 2, 2), 2, 6, 12, 16, 40
PER_SEQ = (1, 3, 6)


def _inputs(seed=3):
    rng = np.random.default_rng(seed)
    w = _tiny_weights(rng, N, E, D, V)
    return w, rng.standard_normal((BATCH, E)), rng.integers(0, V, BATCH)


def _along(w, state, last):
    return lambda q, path: O.logp_along_path(w, state[q], int(last[q]), path, N)


def _as_device(od):
    tables = {"states": [s.copy() for s in od.states], "tok": [t.copy() for t in od.topk_tok],
              "logp": [t.copy() for t in od.topk_logp], "lse": [l.astype(np.float32) for l in od.row_lse]}
    cand = {"tokens": od.cand_tokens.copy(), "scores": od.cand_scores.copy(), "leaf": od.cand_leaf.copy()}
    return tables, cand


def _recompute_candidates(tables, cand):
    lt, ls = O.expand_tree(tables["tok"], tables["logp"], TOP_K, BATCH)
    cand["tokens"], cand["scores"], cand["leaf"] = O.prune(lt, ls, KEEP)


def test_oracle_against_itself_is_an_exact_match():
    w, state, last = _inputs()
    od = O.draft(w, state, last, TOP_K, KEEP, keep_logits=True)
    tables, cand = _as_device(od)
    rep = parity.compare_draft(od, tables, cand, TOP_K, w["head"], along_path=_along(w, state, last))
    assert rep.rows_checked == BATCH * sum(PER_SEQ) and rep.rows_exact == rep.rows_checked
    assert rep.rows_exempt == 0 and rep.cand_exempt == 0 and rep.seqs_cand_identical == BATCH
    assert rep.max_same_input_abs < 1e-6 and rep.max_logp_abs < 1e-6


def test_a_wrong_token_outside_the_band_is_rejected():
    w, state, last = _inputs()
    od = O.draft(w, state, last, TOP_K, KEEP, keep_logits=True)
    tables, cand = _as_device(od)
    # replace the second-best token of a last-stage row by the vocabulary's worst one
    row = od.logits[2][1]
    tables["tok"][2][1][1] = int(np.argmin(row))
    tables["logp"][2][1][1] = np.float32(row.min() - od.row_lse[2][1])
    _recompute_candidates(tables, cand)
    with pytest.raises(AssertionError, match="band"):
        parity.compare_draft(od, tables, cand, TOP_K, w["head"], along_path=_along(w, state, last))


def test_a_swapped_order_outside_the_band_is_rejected():
    w, state, last = _inputs()
    od = O.draft(w, state, last, TOP_K, KEEP, keep_logits=True)
    tables, cand = _as_device(od)
    t, l = tables["tok"][0][0], tables["logp"][0][0]
    assert l[0] - l[1] > 2e-3
    t[[0, 1]] = t[[1, 0]]
    l[[0, 1]] = l[[1, 0]]
    _recompute_candidates(tables, cand)
    with pytest.raises(AssertionError):
        parity.compare_draft(od, tables, cand, TOP_K, w["head"], along_path=_along(w, state, last))


def test_a_drifting_value_is_rejected_although_the_tokens_agree():
    # a log-probability off by 5e-4: no token changes, but it is not what the head gives on that state
    w, state, last = _inputs()
    od = O.draft(w, state, last, TOP_K, KEEP, keep_logits=True)
    tables, cand = _as_device(od)
    tables["logp"][1][2][0] += np.float32(5e-4)
    _recompute_candidates(tables, cand)
    with pytest.raises(AssertionError, match="same state"):
        parity.compare_draft(od, tables, cand, TOP_K, w["head"], along_path=_along(w, state, last))


def test_a_wrong_candidate_cut_is_rejected():
    w, state, last = _inputs()
    od = O.draft(w, state, last, TOP_K, KEEP, keep_logits=True)
    tables, cand = _as_device(od)
    # the device's own tables would prune differently: caught by the bit-exact expand / prune check
    cand["leaf"][0][-1], cand["leaf"][0][-2] = cand["leaf"][0][-2], cand["leaf"][0][-1]
    with pytest.raises(AssertionError, match="own tables"):
        parity.compare_draft(od, tables, cand, TOP_K, w["head"], along_path=_along(w, state, last))


def _device_that_swaps_the_first_two_tokens(w, state, last, od):
    """A stand-in device: takes the two best tokens of sequence 0's first head in the other order and
    builds everything below with the oracle's arithmetic along ITS path."""
    along = _along(w, state, last)
    dev = {"states": [od.states[0].copy()], "tok": [od.topk_tok[0].copy()], "logp": [od.topk_logp[0].copy()],
           "lse": [od.row_lse[0].astype(np.float32)]}
    tok0 = [int(t) for t in od.topk_tok[0][0]]
    tok0[0], tok0[1] = tok0[1], tok0[0]
    dev["tok"][0][0] = tok0
    dev["logp"][0][0] = (od.logits[0][0] - od.row_lse[0][0])[tok0].astype(np.float32)
    for i in (1, 2):
        S, T, LP, LSE = [], [], [], []
        for q in range(BATCH):
            for rl in range(PER_SEQ[i]):
                path, r = [], rl
                for d in range(i, 0, -1):
                    par, rank = r // TOP_K[d - 1], r % TOP_K[d - 1]
                    path.append(int(dev["tok"][d - 1][q * PER_SEQ[d - 1] + par][rank]))
                    r = par
                path.reverse()
                s_o, lp_o = along(q, path)
                idx = O.topk_desc(lp_o.astype(np.float32), TOP_K[i])
                S.append(s_o)
                T.append(idx.astype(np.int32))
                LP.append(lp_o[idx].astype(np.float32))
                LSE.append(np.float32(O.log_softmax(O.head_logits(s_o[None], w["head"][i]))[1][0]))
        dev["states"].append(np.array(S))
        dev["tok"].append(np.array(T))
        dev["logp"].append(np.array(LP))
        dev["lse"].append(np.array(LSE))
    cand = {}
    _recompute_candidates(dev, cand)
    return dev, cand


def _with_first_gap(gap):
    """Inputs whose two best first-head logits of sequence 0 are `gap` apart."""
    w, state, last = _inputs()
    od = O.draft(w, state, last, TOP_K, KEEP, keep_logits=True)
    a, b = int(od.topk_tok[0][0][0]), int(od.topk_tok[0][0][1])
    s, h = od.states[0][0], w["head"][0]
    h[b] += (float(h[a] @ s - h[b] @ s) - gap) * s / float(s @ s)
    od = O.draft(w, state, last, TOP_K, KEEP, keep_logits=True)
    assert (int(od.topk_tok[0][0][0]), int(od.topk_tok[0][0][1])) == (a, b)
    assert abs(float(od.logits[0][0][a] - od.logits[0][0][b]) - gap) < 1e-9
    return w, state, last, od


def test_a_near_tie_inside_the_band_is_exempt_and_the_rows_below_follow_the_device_path():
    w, state, last, od = _with_first_gap(3e-4)
    dev, cand = _device_that_swaps_the_first_two_tokens(w, state, last, od)
    rep = parity.compare_draft(od, dev, cand, TOP_K, w["head"], along_path=_along(w, state, last))
    assert rep.rows_exempt == 1
    assert rep.rows_skipped_below_exempt == PER_SEQ[1] + PER_SEQ[2]      # all of sequence 0 below its first row
    assert rep.rows_checked + rep.rows_skipped_below_exempt == BATCH * sum(PER_SEQ)
    assert rep.seqs_cand_identical == 1


def test_the_same_swap_just_outside_the_band_is_rejected():
    w, state, last, od = _with_first_gap(1.2e-3)
    dev, cand = _device_that_swaps_the_first_two_tokens(w, state, last, od)
    with pytest.raises(AssertionError, match="band"):
        parity.compare_draft(od, dev, cand, TOP_K, w["head"], along_path=_along(w, state, last))
