"""Shared driver of the GPU parity tests: runs one workload through the C ABI
and through the oracle on identical seeded inputs and compares them."""
from __future__ import annotations

import sys
import time
from typing import Optional, Sequence

import numpy as np
import torch

from oracle import spec_oracle as O
from paper_2404_19124_amd import binding as B
from paper_2404_19124_amd import workloads as W
from paper_2404_19124_amd.runner import Step
from tests import parity


def log(msg: str) -> None:
    print("[gpu-test] " + msg, flush=True)
    sys.stdout.flush()


def tables_to_numpy(step: Step):
    t = step.debug_tables()
    return {
        "states": [x.float().cpu().numpy() for x in t["states"]],
        "tok": [x.cpu().numpy() for x in t["tok"]],
        "logp": [x.cpu().numpy() for x in t["logp"]],
        "lse": [x.cpu().numpy() for x in t["lse"]],
    }


def run_workload(wl: W.Workload, ln_affine: str = "identity", gen_device: str = "cuda",
                 sample_seqs: Optional[Sequence[int]] = None, w_s: float = -1.0, w_e: float = -1.0,
                 check_verify: bool = True, tied: bool = False):
    """Returns (report, step, oracle draft, oracle verify)."""
    t0 = time.time()
    log("workload %s: E=%d D=%d V=%d n=%d k=%s B=%d batch=%d dtype=%s seed=%d"
        % (wl.name, wl.emb_dim, wl.inner_dim, wl.vocab, wl.n_predict, wl.top_k, wl.B, wl.batch, wl.weight_dtype, wl.seed))
    gen = W.make_generator(wl.seed, gen_device)
    w = W.make_speculator(wl, gen, device=gen_device, ln_affine=ln_affine)
    if tied:   # weight-tied (RNN-like) variant: stages 2.. share stage 2's tensors (stage 1 has its own input width)
        for key in w:
            for i in range(2, wl.n_predict):
                w[key][i] = w[key][1]
    state, last = W.make_draft_inputs(wl, gen, device=gen_device)
    w_dev = {k: [t.cuda() for t in v] for k, v in w.items()}
    state_d, last_d = state.cuda(), last.cuda()

    step = Step(wl, w_dev, debug=True, state_weight=w_s, emb_weight=w_e)
    step.draft(state_d, last_d)
    torch.cuda.synchronize()
    log("  HIP draft done (%.1fs)" % (time.time() - t0))
    gt = tables_to_numpy(step)
    gc = {"tokens": step.cand_tokens.cpu().numpy(), "scores": step.cand_scores.cpu().numpy(),
          "leaf": step.cand_leaf.cpu().numpy()}

    seqs = list(range(wl.batch)) if sample_seqs is None else list(sample_seqs)
    wn = W.weights_to_numpy(w)
    # (the contraction operands once in float64, so that the oracle's matmuls do not convert them per call)
    wn["head"] = [a.astype(np.float64) for a in wn["head"]]
    wn["proj"] = [a.astype(np.float64) for a in wn["proj"]]
    st_np = W.to_numpy_f32(state)
    lt_np = last.cpu().numpy()
    ms, me, eps = step.model.scalars()
    ows, owe = (None, None) if w_s < 0 else (w_s, w_e)
    if w_s < 0:
        want = O.mix_weights(wl.n_predict)
        assert abs(ms - want[0]) < 1e-6 and abs(me - want[1]) < 1e-6 and abs(eps - 1e-5) < 1e-12

    # the oracle runs the compared sequences in chunks that keep its float64 logit rows bounded (~1.5 GB)
    rows_per_seq = sum(wl.rows()) // wl.batch
    chunk = max(1, min(len(seqs), int(1.5e9 // (8 * rows_per_seq * wl.vocab))))
    rep = parity.Report()
    parts = []
    t1 = time.time()
    for c0 in range(0, len(seqs), chunk):
        sub = seqs[c0:c0 + chunk]
        od_c = O.draft(wn, st_np[sub], lt_np[sub], wl.top_k, wl.B, w_s=ows, w_e=owe, state_dtype=wl.weight_dtype,
                       keep_logits=True)

        def along(q, path, sub=sub):
            return O.logp_along_path(wn, st_np[sub[q]], int(lt_np[sub[q]]), path, wl.n_predict, w_s=ows, w_e=owe,
                                     state_dtype=wl.weight_dtype)

        rep.merge(parity.compare_draft(od_c, gt, gc, wl.top_k, wn["head"], seq_index=sub, along_path=along))
        od_c.logits, od_c.states = [], []
        parts.append(od_c)
        log("  oracle draft + comparison of sequences %d..%d done (%.1fs)" % (sub[0], sub[-1], time.time() - t1))
    od = O.DraftResult(*[np.concatenate([getattr(p, name) for p in parts]) for name in
                         ("cand_tokens", "cand_scores", "cand_leaf", "leaf_tokens", "leaf_scores")])
    assert rep.seqs == len(seqs)
    log("  draft parity (%d of %d sequences): %s" % (len(seqs), wl.batch, rep.line()))
    for note in rep.notes[:5]:
        log("    " + note)

    # The configuration the benchmark times is the one WITHOUT debug outputs.  It must choose the same
    # candidates, and its scores are held to the oracle's leaf scores.
    if w_s < 0 and not tied:
        plain = Step(wl, w_dev)
        plain.draft(state_d, last_d)
        torch.cuda.synchronize()
        assert torch.equal(plain.cand_tokens, step.cand_tokens), "candidates differ between debug and plain run"
        assert torch.equal(plain.cand_leaf, step.cand_leaf)
        p_sc, p_leaf = plain.cand_scores.cpu().numpy().astype(np.float64), plain.cand_leaf.cpu().numpy()
        for g in seqs:
            d = np.abs(p_sc[g] - rep.ref_scores[g][p_leaf[g]]).max()
            assert d <= parity.abs_score(wl.n_predict), "plain run, seq %d: leaf scores off by %.2e from the oracle's" % (g, d)
        plain.close()
        log("  plain (benchmark) configuration: same candidates, scores within the bar of the oracle's")

    ov = None
    if check_verify:
        # candidates fed to both verifies: the oracle's where it ran, seeded random tokens elsewhere
        cand = torch.randint(0, wl.vocab, (wl.batch, wl.B, wl.n_predict), generator=gen, device=gen_device,
                             dtype=torch.int32)
        cand[torch.as_tensor(seqs, device=gen_device)] = torch.from_numpy(od.cand_tokens).to(gen_device)
        logits = W.make_base_logits(wl, cand, gen, device=gen_device)
        cand_d, logits_d = cand.cuda(), logits.cuda()
        step.verify(logits_d, cand_d)
        torch.cuda.synchronize()
        t2 = time.time()
        ov = O.verify(W.to_numpy_f32(logits[torch.as_tensor(seqs, device=logits.device)]), cand.cpu().numpy()[seqs])
        log("  oracle verify done (%.1fs)" % (time.time() - t2))
        compare_verify(step, ov, seqs, wl.n_predict)
        log("  verify parity exact; accepted lengths %s" % np.bincount(ov.accept_len, minlength=wl.n_predict + 1).tolist())
    return rep, step, od, ov


def compare_verify(step: Step, ov: O.VerifyResult, seqs, n: int) -> None:
    g = {k: getattr(step, k).cpu().numpy() for k in ("greedy", "accept_len", "best_cand", "out_tokens", "n_out", "accept_all")}
    assert np.array_equal(g["greedy"][seqs], ov.greedy), "greedy tokens differ"
    assert np.array_equal(g["accept_all"][seqs], ov.accept_all)
    assert np.array_equal(g["accept_len"][seqs], ov.accept_len)
    assert np.array_equal(g["best_cand"][seqs], ov.best_cand)
    assert np.array_equal(g["out_tokens"][seqs], ov.out_tokens)
    assert np.array_equal(g["n_out"][seqs], ov.n_out)
    # properties that hold for every sequence, sampled by the oracle or not
    assert g["accept_len"].min() >= 0 and g["accept_len"].max() <= n
    assert np.array_equal(g["n_out"], g["accept_len"] + 1)
    assert np.array_equal(g["accept_len"], g["accept_all"].max(axis=1))
    assert np.array_equal(g["best_cand"], g["accept_all"].argmax(axis=1))
