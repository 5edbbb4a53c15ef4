"""GPU parity of the per-sequence speculation settings (own tree and candidate count per sequence,
0 = speculation off; Sec. 4.2, 5): spec_draft_dynamic / spec_verify_dynamic through the C ABI
against the oracle's draft_dynamic / verify_dynamic."""
import numpy as np
import pytest
import torch

from oracle import spec_oracle as O
from paper_2404_19124_amd import binding as B
from paper_2404_19124_amd import workloads as W
from paper_2404_19124_amd.runner import Step
from tests import parity
from tests.gpu_common import log

pytestmark = pytest.mark.gpu


def _run_dynamic(wl, w_dev, state, last, top_k_seq, B_seq, B_pad, debug=True):
    """One spec_draft_dynamic call; returns the outputs and, with debug, per-stage device tables."""
    batch, n, D = wl.batch, wl.n_predict, wl.inner_dim
    step = Step(wl, w_dev, max_batch=batch, max_top_k=wl.top_k)
    i32 = dict(dtype=torch.int32, device="cuda")
    out = {"tokens": torch.full((batch, B_pad, n), 77, **i32), "scores": torch.full((batch, B_pad), 7.0, device="cuda"),
           "leaf": torch.full((batch, B_pad), 77, **i32), "n_cand": torch.full((batch,), 77, **i32)}
    rows, kw, first = B.dynamic_rows(top_k_seq, B_seq)
    dbg = None
    if debug:
        sdt = torch.bfloat16 if wl.weight_dtype == "bf16" else torch.float32
        sum_rows, sum_rk = sum(rows), sum(r * k for r, k in zip(rows, kw))
        dbg = {"stage_state": torch.zeros((sum_rows, D), dtype=sdt, device="cuda"),
               "topk_tok": torch.zeros((sum_rk,), **i32), "topk_logp": torch.zeros((sum_rk,), device="cuda"),
               "row_lse": torch.zeros((sum_rows,), device="cuda")}
    B.spec_draft_dynamic(step.model, state, last, top_k_seq, B_seq, out["tokens"], out["scores"], out["leaf"],
                         out["n_cand"], dbg)
    torch.cuda.synchronize()
    tables = None
    if debug:
        tables = {"states": [], "tok": [], "logp": [], "lse": []}
        ro = ko = 0
        for r, k in zip(rows, kw):
            tables["states"].append(dbg["stage_state"][ro:ro + r].float().cpu().numpy())
            tables["lse"].append(dbg["row_lse"][ro:ro + r].cpu().numpy())
            tables["tok"].append(dbg["topk_tok"][ko:ko + r * k].view(r, k).cpu().numpy())
            tables["logp"].append(dbg["topk_logp"][ko:ko + r * k].view(r, k).cpu().numpy())
            ro += r
            ko += r * k
    return step, {k: v.cpu().numpy() for k, v in out.items()}, tables, first


def _compare_with_oracle(wl, w, state, last, top_k_seq, B_seq, B_pad, got, tables, first):
    wn = W.weights_to_numpy(w)
    st_np, lt_np = W.to_numpy_f32(state), last.cpu().numpy()
    od = O.draft_dynamic(wn, st_np, lt_np, top_k_seq, B_seq, B_pad, state_dtype=wl.weight_dtype)
    assert np.array_equal(got["n_cand"], od["n_cand"])
    total = parity.Report()
    for q, (ks, Bq) in enumerate(zip(top_k_seq, B_seq)):
        # padding behind the sequence's candidates, bit for bit
        assert (got["tokens"][q, Bq:] == -1).all() and (got["leaf"][q, Bq:] == -1).all()
        assert np.isneginf(got["scores"][q, Bq:]).all()
        if Bq == 0:
            continue
        # this sequence's rows of the device tables, cut to its own branching
        cnt, tq = 1, {"states": [], "tok": [], "logp": [], "lse": []}
        for i, k in enumerate(ks):
            r0 = first[q][i]
            tq["states"].append(tables["states"][i][r0:r0 + cnt])
            tq["lse"].append(tables["lse"][i][r0:r0 + cnt])
            tq["tok"].append(tables["tok"][i][r0:r0 + cnt, :k])
            tq["logp"].append(tables["logp"][i][r0:r0 + cnt, :k])
            cnt *= k
        cq = {"tokens": got["tokens"][q:q + 1, :Bq], "scores": got["scores"][q:q + 1, :Bq],
              "leaf": got["leaf"][q:q + 1, :Bq]}

        def along(_, path, q=q):
            return O.logp_along_path(wn, st_np[q], int(lt_np[q]), path, wl.n_predict, state_dtype=wl.weight_dtype)

        total.merge(parity.compare_draft(od["per_seq"][q], tq, cq, ks, wn["head"], along_path=along))
    log("  dynamic draft parity: " + total.line())
    return od, total


MIXED = [
    # name, E, D, V, n, max_top_k, batch, dtype, top_k_seq, B_seq, B_pad
    ("skinny_mixed", 128, 192, 1000, 3, (4, 3, 2), 4, "bf16",
     [(4, 3, 1), (1, 1, 1), (1, 1, 1), (2, 1, 2)], [5, 1, 0, 4], 6),                   # 3, 7, 14 rows
    ("dense_mixed", 256, 128, 2049, 3, (5, 3, 2), 9, "bf16",
     [(5, 3, 2), (1, 1, 1), (2, 2, 2), (1, 1, 1), (5, 1, 1), (3, 3, 2), (1, 1, 1), (4, 2, 1), (2, 3, 2)],
     [16, 1, 8, 0, 3, 10, 0, 8, 12], 16),                                               # 7, 23, 48 rows
    ("f32_mixed", 100, 72, 333, 3, (3, 3, 2), 5, "f32",
     [(3, 3, 2), (1, 1, 1), (1, 2, 1), (2, 2, 2), (3, 1, 1)], [7, 0, 2, 8, 1], 8),
    ("first_sequence_off", 64, 64, 300, 2, (3, 2), 3, "bf16", [(1, 1), (3, 2), (2, 1)], [0, 6, 1], 6),
]


@pytest.mark.parametrize("case", MIXED, ids=[c[0] for c in MIXED])
def test_mixed_batch_of_off_chain_and_tree_sequences(case):
    name, E, D, V, n, max_k, batch, dtype, top_k_seq, B_seq, B_pad = case
    wl = W.Workload(name, E, D, V, n, max_k, B_pad, batch, dtype, "f32", 0.6, seed=41, emb_std=0.3)
    log("dynamic %s: top_k %s B %s" % (name, top_k_seq, B_seq))
    gen = W.make_generator(wl.seed)
    w = W.make_speculator(wl, gen, ln_affine="random")
    state, last = W.make_draft_inputs(wl, gen)
    w_dev = {k: [t.cuda() for t in v] for k, v in w.items()}
    step, got, tables, first = _run_dynamic(wl, w_dev, state.cuda(), last.cuda(), top_k_seq, B_seq, B_pad)
    od, rep = _compare_with_oracle(wl, w, state, last, top_k_seq, B_seq, B_pad, got, tables, first)
    assert rep.seqs == sum(1 for x in B_seq if x > 0) and rep.rows_exempt <= 1
    rows, _, _ = B.dynamic_rows(top_k_seq, B_seq)
    assert rep.rows_checked + rep.rows_skipped_below_exempt == sum(rows)
    # the run without debug outputs writes the same candidates
    step2, got2, _, _ = _run_dynamic(wl, w_dev, state.cuda(), last.cuda(), top_k_seq, B_seq, B_pad, debug=False)
    for key in ("tokens", "scores", "leaf", "n_cand"):
        assert np.array_equal(got[key], got2[key]), key

    # ---- verify on these candidates: padding rows of the logits are poisoned, they must never be read
    cand = torch.from_numpy(od["cand_tokens"])
    real = cand >= 0
    safe = torch.where(real, cand, torch.zeros_like(cand))
    logits = W.make_base_logits(wl, safe, gen)
    ncand = torch.tensor(B_seq, dtype=torch.int32)
    for q, Bq in enumerate(B_seq):
        logits[q, max(Bq, 1):] = float("nan")
        if Bq == 0:
            logits[q, 0, 1:] = float("nan")
    i32 = dict(dtype=torch.int32, device="cuda")
    v = {"greedy": torch.full((batch, B_pad, n + 1), 55, **i32), "accept_len": torch.full((batch,), 55, **i32),
         "best_cand": torch.full((batch,), 55, **i32), "out_tokens": torch.full((batch, n + 1), 55, **i32),
         "n_out": torch.full((batch,), 55, **i32), "accept_all": torch.full((batch, B_pad), 55, **i32)}
    B.spec_verify_dynamic(logits.cuda(), torch.from_numpy(got["tokens"]).cuda(), torch.from_numpy(got["n_cand"]).cuda(),
                          v["greedy"], v["accept_len"], v["best_cand"], v["out_tokens"], v["n_out"], v["accept_all"])
    torch.cuda.synchronize()
    ov = O.verify_dynamic(np.nan_to_num(logits.numpy(), nan=-1e30), got["tokens"], got["n_cand"])
    for key in ("greedy", "accept_len", "best_cand", "out_tokens", "n_out", "accept_all"):
        assert np.array_equal(v[key].cpu().numpy(), getattr(ov, key)), key
    off = [q for q, Bq in enumerate(B_seq) if Bq == 0]
    assert (ov.n_out[off] == 1).all() and (ov.out_tokens[off, 0] >= 0).all()
    log("  dynamic verify exact; accepted lengths %s" % ov.accept_len.tolist())
    step.close()
    step2.close()


def test_uniform_settings_reproduce_spec_draft_bit_for_bit_and_all_off_gives_padding():
    wl = W.Workload("dyn_uniform", 256, 128, 2049, 3, (5, 3, 2), 16, 7, "bf16", "f32", 0.6, seed=43, emb_std=0.3)
    gen = W.make_generator(wl.seed)
    w_dev = {k: [t.cuda() for t in v] for k, v in W.make_speculator(wl, gen, ln_affine="random").items()}
    state, last = W.make_draft_inputs(wl, gen)
    state, last = state.cuda(), last.cuda()
    ref = Step(wl, w_dev)
    ref.draft(state, last)
    torch.cuda.synchronize()
    _, got, _, _ = _run_dynamic(wl, w_dev, state, last, [wl.top_k] * wl.batch, [wl.B] * wl.batch, wl.B, debug=False)
    assert np.array_equal(got["tokens"], ref.cand_tokens.cpu().numpy())
    assert np.array_equal(got["scores"], ref.cand_scores.cpu().numpy())
    assert np.array_equal(got["leaf"], ref.cand_leaf.cpu().numpy())
    # every sequence off: no row at all, outputs are padding, and verify returns the base model's tokens
    _, off, _, _ = _run_dynamic(wl, w_dev, state, last, [wl.top_k] * wl.batch, [0] * wl.batch, 4, debug=False)
    assert (off["tokens"] == -1).all() and (off["leaf"] == -1).all() and np.isneginf(off["scores"]).all()
    assert (off["n_cand"] == 0).all()
    ref.close()


def test_llama7b_shape_with_speculation_off_for_part_of_the_batch():
    """The 7B-shaped model with 16 sequences: a quarter speculates with the 5/3/2 tree, half with a k = 1
    chain, a quarter not at all; oracle on the speculating sequences."""
    base = W.WORKLOADS["llama7b_b64"]
    wl = W.small_variant(base, name="llama7b_dyn_b16", batch=16)
    gen = W.make_generator(wl.seed, "cuda")
    w = W.make_speculator(wl, gen, device="cuda")
    state, last = W.make_draft_inputs(wl, gen, device="cuda")
    top_k_seq = [(5, 3, 2) if q % 4 == 0 else (1, 1, 1) for q in range(16)]
    B_seq = [16 if q % 4 == 0 else (0 if q % 4 == 3 else 1) for q in range(16)]
    step, got, tables, first = _run_dynamic(wl, w, state, last, top_k_seq, B_seq, 16)
    od, rep = _compare_with_oracle(wl, w, state, last, top_k_seq, B_seq, 16, got, tables, first)
    assert rep.seqs == 12 and rep.rows_checked + rep.rows_skipped_below_exempt == 4 * 21 + 8 * 3
    assert rep.rows_exempt <= 2
    step.close()


def test_dynamic_draft_rejects_bad_arguments():
    wl = W.Workload("dyn_err", 64, 64, 100, 2, (3, 2), 6, 2, "bf16", "f32", 0.5)
    gen = W.make_generator(0)
    w_dev = {k: [t.cuda() for t in v] for k, v in W.make_speculator(wl, gen).items()}
    state, last = W.make_draft_inputs(wl, gen)
    step = Step(wl, w_dev)
    i32 = dict(dtype=torch.int32, device="cuda")
    out = (torch.zeros((2, 6, 2), **i32), torch.zeros((2, 6), device="cuda"), torch.zeros((2, 6), **i32),
           torch.zeros((2,), **i32))
    with pytest.raises(B.SpecError) as e:      # more candidates than the sequence's tree has leaves
        B.spec_draft_dynamic(step.model, state.cuda(), last.cuda(), [(3, 2), (1, 1)], [6, 2], *out)
    assert e.value.status == B.SPEC_EINVAL
    with pytest.raises(B.SpecError) as e:      # branching above what the model was created for
        B.spec_draft_dynamic(step.model, state.cuda(), last.cuda(), [(4, 2), (1, 1)], [6, 1], *out)
    assert e.value.status == B.SPEC_ESHAPE
    with pytest.raises(B.SpecError) as e:      # more candidates than output slots
        B.spec_draft_dynamic(step.model, state.cuda(), last.cuda(), [(3, 2), (3, 2)], [6, 6],
                             torch.zeros((2, 4, 2), **i32), torch.zeros((2, 4), device="cuda"),
                             torch.zeros((2, 4), **i32), out[3])
    assert e.value.status == B.SPEC_EINVAL
    with pytest.raises(ValueError):
        B.spec_draft_dynamic(step.model, state.cuda(), last.cuda(), [(3, 2)], [6, 6], *out)
    # the settings of a switched-off sequence are not read
    B.spec_draft_dynamic(step.model, state.cuda(), last.cuda(), [(99, 99), (3, 2)], [0, 6], *out)
    torch.cuda.synchronize()
    assert (out[0][0] == -1).all() and (out[0][1] >= 0).all()
    step.close()
