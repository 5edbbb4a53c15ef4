"""CPU oracle for one speculative-decoding draft + verify step of the combined
token/embedding speculator (arXiv 2404.19124).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke check
and the CPU-baseline leg of the benchmark may import it.  It shares no code with
the HIP library and never calls it.  It is written to be checked against the
paper by eye: plain numpy in float64, one function per step of the method, taken
in the order the paper states them, with a library matmul / erf / sort as the
only primitives.  No blocking, fusion or reordering.

What the paper fixes (cited per function below):
  * Sec. 3.1: a multi-stage MLP; stage i takes the previous state vector and the
    embedding of the token sampled by the previous stage (the base model is
    stage 0), projects the pair, applies LayerNorm then GELU, giving the new
    state; that state predicts the next draft tokens and feeds stage i+1.  The
    stages emit a tree of candidates, from which the top-k most likely are kept.
  * Sec. 4: latent width 4096; state / embedding projections are weighted so
    that the base model's state carries 50% of the variance of the state at the
    last head, in expectation.
  * Sec. 4.1: per-head branching (6, 3, 2 -> 36 leaves), pruned to the wanted
    number of candidates by confidence; greedy inference.
  * Sec. 1 and 3.1: verification compares the base model's outputs with the
    speculated inputs, accepts the matching tokens, and keeps the tokens of the
    best candidate only.
  * Sec. 4.1 and 5: each candidate is n+1 tokens long (one token from the base
    model plus n speculated); a step emits at most n accepted tokens plus one
    base-model ("bonus") token.

Where the paper is silent, the readings taken here (each also listed in the
design notes of this repository):
  - the pair is combined as  z = w_s * (W_i s) + w_e * Emb_i[t]   (two weighted
    projections; the embedding lookup is the projection of a one-hot token);
  - no biases; LayerNorm over the latent dimension, biased variance, eps inside
    the square root, affine gamma / beta; GELU is the exact erf form;
  - confidence of a leaf = sum over stages of the natural-log softmax
    probability of its tokens; only leaves are pruned (no per-level beam);
  - ties: larger value first, then smaller index (token id, leaf index,
    candidate index, vocabulary index);
  - bf16 configurations: weights, embeddings and the input state are bf16
    values; the new state of each stage is rounded once to bf16 and that rounded
    value feeds both the head and the next projection; everything else is not
    rounded.  Top-k and pruning decisions are taken on float32-rounded logits
    and scores, the precision the device path decides in.

Parity pins (tests/test_oracle_*.py): every function here is pinned to a closed
form, a library routine, a brute-force enumeration or an invariant.  Behaviour
of *trained* speculators (the paper's tokens-per-step figures) is "parity
unpinned": it needs the released weights and base models, which are not here.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


# --------------------------------------------------------------------------
# scalar rules
# --------------------------------------------------------------------------
def mix_weights(n_predict: int) -> tuple:
    """(w_s, w_e) from the 50%-variance rule of Sec. 4.

    With unit-variance, uncorrelated inputs and w_s^2 + w_e^2 = 1 the state keeps
    unit variance, and the share of the base state after n stages is w_s^(2n).
    Setting that to 1/2 gives the closed form below.
    """
    w_s = 0.5 ** (1.0 / (2.0 * n_predict))
    w_e = math.sqrt(1.0 - 0.5 ** (1.0 / n_predict))
    return w_s, w_e


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bfloat16 (8 significant bits), ties to
    even, returned as float64.  Subnormal / overflow ranges are not treated: the
    states this is applied to are O(1)."""
    x = np.asarray(x, dtype=F64)
    m, e = np.frexp(x)                      # x = m * 2**e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0), e - 8)   # np.rint rounds half to even


# --------------------------------------------------------------------------
# one stage (Sec. 3.1)
# --------------------------------------------------------------------------
def project(s_prev: np.ndarray, W: np.ndarray) -> np.ndarray:
    """State projection  W s  for each row of s_prev.  W is [D, in] (out, in)."""
    return np.asarray(s_prev, F64) @ np.asarray(W, F64).T


def layer_norm(z: np.ndarray, gamma: np.ndarray, beta: np.ndarray, eps: float) -> np.ndarray:
    """LayerNorm over the last axis: biased variance, eps inside the root."""
    z = np.asarray(z, F64)
    mu = z.mean(axis=-1, keepdims=True)
    var = ((z - mu) ** 2).mean(axis=-1, keepdims=True)
    return (z - mu) / np.sqrt(var + eps) * np.asarray(gamma, F64) + np.asarray(beta, F64)


def gelu(x: np.ndarray) -> np.ndarray:
    """Exact GELU:  x * Phi(x)  with Phi the standard normal CDF."""
    x = np.asarray(x, F64)
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))


def stage_state(pz_parent: np.ndarray, emb_rows: np.ndarray, gamma, beta,
                w_s: float, w_e: float, eps: float, state_dtype: str) -> np.ndarray:
    """New state of a stage from the projected parent state and the embedding of
    the token that node carries:  GELU(LN(w_s * Wz + w_e * e)), rounded to the
    storage type of the configuration."""
    z = w_s * np.asarray(pz_parent, F64) + w_e * np.asarray(emb_rows, F64)
    s = gelu(layer_norm(z, gamma, beta, eps))
    if state_dtype == "bf16":
        s = round_bf16(s)
    elif state_dtype != "f32":
        raise ValueError("state_dtype must be 'f32' or 'bf16'")
    return s


def head_logits(s: np.ndarray, H: np.ndarray) -> np.ndarray:
    """Vocabulary head: one logit per vocabulary entry.  H is [V, D]."""
    return np.asarray(s, F64) @ np.asarray(H, F64).T


def log_softmax(logits: np.ndarray):
    """Natural-log softmax over the last axis; returns (logp, lse)."""
    logits = np.asarray(logits, F64)
    m = logits.max(axis=-1, keepdims=True)
    lse = m + np.log(np.exp(logits - m).sum(axis=-1, keepdims=True))
    return logits - lse, lse[..., 0]


def topk_desc(values: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest entries of a 1-D array, largest first; equal
    values keep the smaller index first."""
    order = np.argsort(-np.asarray(values), kind="stable")
    return order[:k]


# --------------------------------------------------------------------------
# draft
# --------------------------------------------------------------------------
@dataclass
class DraftResult:
    cand_tokens: np.ndarray          # [b, B, n] int32
    cand_scores: np.ndarray          # [b, B] float32, descending
    cand_leaf: np.ndarray            # [b, B] int32, leaf index in mixed-radix order
    leaf_tokens: np.ndarray          # [b, L, n] int32
    leaf_scores: np.ndarray          # [b, L] float32
    states: List[np.ndarray] = field(default_factory=list)     # per stage [R_i, D] float64
    topk_tok: List[np.ndarray] = field(default_factory=list)   # per stage [R_i, k_i] int32
    topk_logp: List[np.ndarray] = field(default_factory=list)  # per stage [R_i, k_i] float32
    row_lse: List[np.ndarray] = field(default_factory=list)    # per stage [R_i] float64
    logits: List[np.ndarray] = field(default_factory=list)     # per stage [R_i, V] float64 (optional)


def draft(weights: dict, state: np.ndarray, last_tok: np.ndarray, top_k: Sequence[int], B: int,
          w_s: Optional[float] = None, w_e: Optional[float] = None, eps: float = 1e-5,
          state_dtype: str = "f32", keep_logits: bool = False) -> DraftResult:
    """The draft half of a step (Sec. 3.1, 4.1).

    weights: dict of per-stage lists  proj[i] [D, in_i], emb[i] [V, D],
             head[i] [V, D], ln_gamma[i] [D], ln_beta[i] [D]   (in_1 = E, else D)
    state [b, E]: the base model's last hidden vector; last_tok [b]: the token
    the base model just sampled.  top_k[i]: branches of stage i; B: candidates kept.

    Rows of a stage are ordered  sequence-major, then by the ranks chosen at the
    earlier stages (mixed radix), so node r at depth i-1 has children
    r*k_i + j,  j = 0..k_i-1, and parent r // k_{i-1}.
    """
    n = len(top_k)
    b = state.shape[0]
    if w_s is None or w_e is None:
        w_s, w_e = mix_weights(n)
    L = int(np.prod(top_k))
    if not (1 <= B <= L):
        raise ValueError("B must be in [1, prod(top_k)]")

    res = DraftResult(None, None, None, None, None)
    s_prev = np.asarray(state, F64)                 # parent states of stage 1: one per sequence
    node_tok = np.asarray(last_tok).astype(np.int64)  # token carried by each node at depth i-1
    k_prev = 1
    for i in range(n):
        pz = project(s_prev, weights["proj"][i])                     # one row per distinct parent
        parent = np.arange(node_tok.shape[0]) // k_prev              # siblings share the parent state
        e = np.asarray(weights["emb"][i][node_tok], F64)            # embedding rows of the carried tokens
        s = stage_state(pz[parent], e, weights["ln_gamma"][i], weights["ln_beta"][i],
                        w_s, w_e, eps, state_dtype)
        logits = head_logits(s, weights["head"][i])
        logp, lse = log_softmax(logits)
        decide = logits.astype(np.float32)                           # decision precision
        k_i = int(top_k[i])
        tok = np.empty((s.shape[0], k_i), np.int32)
        lp = np.empty((s.shape[0], k_i), np.float32)
        for r in range(s.shape[0]):
            idx = topk_desc(decide[r], k_i)
            tok[r] = idx
            lp[r] = logp[r, idx].astype(np.float32)
        res.states.append(s)
        res.topk_tok.append(tok)
        res.topk_logp.append(lp)
        res.row_lse.append(lse)
        if keep_logits:
            res.logits.append(logits)
        s_prev = s
        node_tok = tok.reshape(-1).astype(np.int64)
        k_prev = k_i

    res.leaf_tokens, res.leaf_scores = expand_tree(res.topk_tok, res.topk_logp, top_k, b)
    res.cand_tokens, res.cand_scores, res.cand_leaf = prune(res.leaf_tokens, res.leaf_scores, B)
    return res


def expand_tree(topk_tok, topk_logp, top_k: Sequence[int], b: int):
    """All prod(k_i) leaves of each sequence's tree, in mixed-radix order of the
    per-stage ranks (first stage most significant).  The score of a leaf is the
    sum of its tokens' log-probabilities, added in stage order in float32."""
    n = len(top_k)
    L = int(np.prod(top_k))
    leaf_tokens = np.empty((b, L, n), np.int32)
    leaf_scores = np.empty((b, L), np.float32)
    for q in range(b):
        for leaf in range(L):
            # ranks j_1..j_n of this leaf
            ranks, rem = [], leaf
            for i in reversed(range(n)):
                ranks.append(rem % top_k[i])
                rem //= top_k[i]
            ranks.reverse()
            score = np.float32(0.0)
            row = q                       # row of stage 1 for this sequence
            for i in range(n):
                leaf_tokens[q, leaf, i] = topk_tok[i][row, ranks[i]]
                score = np.float32(score + topk_logp[i][row, ranks[i]])
                row = row * top_k[i] + ranks[i]      # child row at the next stage
            leaf_scores[q, leaf] = score
    return leaf_tokens, leaf_scores


def prune(leaf_tokens: np.ndarray, leaf_scores: np.ndarray, B: int):
    """Keep the B most confident leaves of each sequence, most confident first;
    equal scores keep the smaller leaf index first (Sec. 4.1)."""
    b, L, n = leaf_tokens.shape
    cand_tokens = np.empty((b, B, n), np.int32)
    cand_scores = np.empty((b, B), np.float32)
    cand_leaf = np.empty((b, B), np.int32)
    for q in range(b):
        keep = topk_desc(leaf_scores[q], B)
        cand_leaf[q] = keep
        cand_scores[q] = leaf_scores[q, keep]
        cand_tokens[q] = leaf_tokens[q, keep]
    return cand_tokens, cand_scores, cand_leaf


# --------------------------------------------------------------------------
# verify
# --------------------------------------------------------------------------
@dataclass
class VerifyResult:
    accept_len: np.ndarray   # [b] in [0, n]
    best_cand: np.ndarray    # [b] in [0, B)
    out_tokens: np.ndarray   # [b, n+1], accepted tokens then the bonus token, rest -1
    n_out: np.ndarray        # [b] = accept_len + 1
    greedy: np.ndarray       # [b, B, n+1] base model's greedy token at each position
    accept_all: np.ndarray   # [b, B] accepted length of every candidate


def verify(base_logits: np.ndarray, cand_tokens: np.ndarray) -> VerifyResult:
    """The verify half of a step (Sec. 1, 3.1, 4.1, 5), greedy.

    base_logits [b, B, n+1, V]: position p of candidate c holds the base model's
    output after consuming (last token, cand[c, :p]); so its greedy token is
    what the base model itself would emit at draft position p.  A candidate's
    accepted length is the number of leading positions where that greedy token
    equals the speculated one.  The best candidate is the one with the longest
    accepted length (first such).  Output = its accepted tokens followed by the
    base model's own token at the first position not accepted (the bonus token;
    position n when everything was accepted)."""
    b, B, n1, V = base_logits.shape
    n = n1 - 1
    assert cand_tokens.shape == (b, B, n)
    greedy = np.empty((b, B, n1), np.int32)
    accept_all = np.empty((b, B), np.int32)
    accept_len = np.empty((b,), np.int32)
    best_cand = np.empty((b,), np.int32)
    out_tokens = np.full((b, n1), -1, np.int32)
    for q in range(b):
        for c in range(B):
            for p in range(n1):
                greedy[q, c, p] = int(np.argmax(base_logits[q, c, p]))   # first maximum
            a = 0
            while a < n and greedy[q, c, a] == cand_tokens[q, c, a]:
                a += 1
            accept_all[q, c] = a
        best = int(np.argmax(accept_all[q]))                              # first longest
        a = int(accept_all[q, best])
        best_cand[q] = best
        accept_len[q] = a
        out_tokens[q, :a] = cand_tokens[q, best, :a]
        out_tokens[q, a] = greedy[q, best, a]
    return VerifyResult(accept_len, best_cand, out_tokens, accept_len + 1, greedy, accept_all)


# --------------------------------------------------------------------------
# validator form: the oracle followed along a path somebody else chose
# --------------------------------------------------------------------------
def logp_along_path(weights: dict, state_row: np.ndarray, last_tok: int, path: Sequence[int],
                    n_predict: int, w_s: Optional[float] = None, w_e: Optional[float] = None,
                    eps: float = 1e-5, state_dtype: str = "f32"):
    """Follow one root-to-node path.  `path` holds the tokens chosen at stages
    1..len(path); returns (state, logp row) of stage len(path)+1, i.e. the
    distribution from which that node's children are drawn.  `n_predict` fixes
    the default mix weights.  Used to brute-force trees and to judge a tree
    whose near-tied choices differ from the oracle's own."""
    if w_s is None or w_e is None:
        w_s, w_e = mix_weights(n_predict)
    s = np.asarray(state_row, F64)[None, :]
    toks = [int(last_tok)] + [int(t) for t in path]
    logp = None
    for i, t in enumerate(toks):
        pz = project(s, weights["proj"][i])
        e = np.asarray(weights["emb"][i][[t]], F64)
        s = stage_state(pz, e, weights["ln_gamma"][i], weights["ln_beta"][i], w_s, w_e, eps, state_dtype)
        logp, _ = log_softmax(head_logits(s, weights["head"][i]))
    return s[0], logp[0]


# ---------------------------------------------------------------------------
# Widening beyond one step: token tree of the candidates, and the hand-over to
# the next step.
# ---------------------------------------------------------------------------
def tree_metadata(cand_tokens: np.ndarray) -> dict:
    """Sec. 3.1 (multi-candidate decoding with tree attention): the B candidates of a
    sequence are root-to-leaf paths that share prefixes; a base model that evaluates
    them as ONE tree needs every distinct prefix once.  The paper names the technique
    only; the encoding is this build's (bit-exact contract with the device):

      * a node = a distinct prefix cand[c, :p+1]; nodes are numbered in order of first
        appearance when the candidates are scanned c = 0..B-1, p = 0..n-1;
      * node_tok = last token of the prefix, node_depth = p + 1, node_parent = node of
        the prefix one shorter (-1 at depth 1: the parent is the sequence's last real token);
      * cand_node[c, p] = node of cand[c, :p+1];
      * mask[i, j] = 1 iff node j is node i or one of its ancestors.
    Arrays are sized M = B * n per sequence; unused entries are -1 (0 for depth, mask).
    """
    cand = np.asarray(cand_tokens)
    b, B, n = cand.shape
    M = B * n
    out = {
        "node_tok": np.full((b, M), -1, np.int32), "node_parent": np.full((b, M), -1, np.int32),
        "node_depth": np.zeros((b, M), np.int32), "n_nodes": np.zeros((b,), np.int32),
        "cand_node": np.full((b, B, n), -1, np.int32), "mask": np.zeros((b, M, M), np.uint8),
    }
    for q in range(b):
        seen = {}
        for c in range(B):
            for p in range(n):
                key = tuple(int(t) for t in cand[q, c, :p + 1])
                if key not in seen:
                    i = len(seen)
                    seen[key] = i
                    out["node_tok"][q, i] = key[-1]
                    out["node_depth"][q, i] = p + 1
                    out["node_parent"][q, i] = -1 if p == 0 else seen[key[:-1]]
                out["cand_node"][q, c, p] = seen[key]
        out["n_nodes"][q] = len(seen)
        for i in range(len(seen)):
            j = i
            while j >= 0:
                out["mask"][q, i, j] = 1
                j = int(out["node_parent"][q, j])
    return out


def advance(hidden: np.ndarray, best_cand: np.ndarray, accept_len: np.ndarray, out_tokens: np.ndarray):
    """Sec. 3.1 (the base model is stage 0 of the next draft): the next step starts from the
    base model's state vector at the last position whose prediction was kept, i.e. position
    a = accept_len of the best candidate, and from the token predicted there (the bonus token,
    out_tokens[a]).  hidden [b, B, n+1, E] -> (next_state [b, E], next_tok [b])."""
    hidden = np.asarray(hidden)
    b = hidden.shape[0]
    idx = np.arange(b)
    a = np.asarray(accept_len).astype(np.int64)
    return hidden[idx, np.asarray(best_cand).astype(np.int64), a, :].copy(), \
        np.asarray(out_tokens)[idx, a].astype(np.int32)


# ---------------------------------------------------------------------------
# Per-sequence speculation settings (Sec. 4.2: speculation is switched off
# dynamically above a batch size; Sec. 5: the number of candidates is swapped
# dynamically to the best value for each incoming request).
# ---------------------------------------------------------------------------
def draft_dynamic(weights: dict, state: np.ndarray, last_tok: np.ndarray, top_k_seq, B_seq, B_pad: int,
                  w_s: Optional[float] = None, w_e: Optional[float] = None, eps: float = 1e-5,
                  state_dtype: str = "f32"):
    """The draft with its own tree per sequence: top_k_seq[q][i] branches at stage i and B_seq[q]
    candidates kept for sequence q; B_seq[q] = 0 switches speculation off for that sequence (it has
    no candidates; the step then emits only the base model's own token).  Sequences do not interact,
    so sequence q's candidates are those of the plain draft run on q alone with q's settings.  The
    mix weights follow the MODEL (n stages), whatever a sequence's tree looks like.

    Outputs are padded to B_pad candidates: cand_tokens [b, B_pad, n] (-1), cand_scores [b, B_pad]
    (-inf), cand_leaf [b, B_pad] (-1), n_cand [b] = B_seq; `per_seq` holds each active sequence's
    full DraftResult."""
    state = np.asarray(state)
    b = state.shape[0]
    top_k_seq = np.asarray(top_k_seq, np.int64).reshape(b, -1)
    n = top_k_seq.shape[1]
    B_seq = np.asarray(B_seq, np.int64).reshape(b)
    if w_s is None or w_e is None:
        w_s, w_e = mix_weights(n)
    if B_seq.max(initial=0) > B_pad:
        raise ValueError("B_pad is smaller than the largest B_seq")
    cand_tokens = np.full((b, B_pad, n), -1, np.int32)
    cand_scores = np.full((b, B_pad), -np.inf, np.float32)
    cand_leaf = np.full((b, B_pad), -1, np.int32)
    per_seq = [None] * b
    for q in range(b):
        Bq = int(B_seq[q])
        if Bq == 0:
            continue                                   # speculation off
        r = draft(weights, state[q:q + 1], np.asarray(last_tok)[q:q + 1], [int(k) for k in top_k_seq[q]], Bq,
                  w_s=w_s, w_e=w_e, eps=eps, state_dtype=state_dtype, keep_logits=True)
        cand_tokens[q, :Bq] = r.cand_tokens[0]
        cand_scores[q, :Bq] = r.cand_scores[0]
        cand_leaf[q, :Bq] = r.cand_leaf[0]
        per_seq[q] = r
    return {"cand_tokens": cand_tokens, "cand_scores": cand_scores, "cand_leaf": cand_leaf,
            "n_cand": B_seq.astype(np.int32), "per_seq": per_seq}


def verify_dynamic(base_logits: np.ndarray, cand_tokens: np.ndarray, n_cand: np.ndarray) -> VerifyResult:
    """Verification when sequence q has only n_cand[q] candidates (the rest of its B slots is padding).
    With n_cand[q] >= 1 it is verify() over q's first n_cand[q] candidates.  With n_cand[q] = 0
    (speculation off) the base model ran an ordinary decoding step: only base_logits[q, 0, 0] exists, its
    greedy token is the step's one output (accept_len 0, n_out 1).  Positions that were not evaluated have
    greedy = -1 and accept_all = 0."""
    b, B, n1, V = base_logits.shape
    n = n1 - 1
    greedy = np.full((b, B, n1), -1, np.int32)
    accept_all = np.zeros((b, B), np.int32)
    accept_len = np.zeros((b,), np.int32)
    best_cand = np.zeros((b,), np.int32)
    out_tokens = np.full((b, n1), -1, np.int32)
    for q in range(b):
        nc = int(n_cand[q])
        if nc == 0:
            greedy[q, 0, 0] = int(np.argmax(base_logits[q, 0, 0]))
            out_tokens[q, 0] = greedy[q, 0, 0]
            continue
        r = verify(base_logits[q:q + 1, :nc], cand_tokens[q:q + 1, :nc])
        greedy[q, :nc] = r.greedy[0]
        accept_all[q, :nc] = r.accept_all[0]
        accept_len[q] = r.accept_len[0]
        best_cand[q] = r.best_cand[0]
        out_tokens[q] = r.out_tokens[0]
    return VerifyResult(accept_len, best_cand, out_tokens, accept_len + 1, greedy, accept_all)
