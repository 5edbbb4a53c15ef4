"""GPU parity of the rows beyond one step: token-tree metadata of the candidates and
the device-side hand-over that chains steps without a host round trip."""
import numpy as np
import pytest
import torch

from oracle import spec_oracle as O
from paper_2404_19124_amd import binding as B
from paper_2404_19124_amd import workloads as W
from paper_2404_19124_amd.runner import Step
from tests import parity
from tests.gpu_common import log, tables_to_numpy

pytestmark = pytest.mark.gpu


def _device_metadata(cand: torch.Tensor, with_mask=True):
    b, Bc, n = cand.shape
    M = Bc * n
    i32 = dict(dtype=torch.int32, device="cuda")
    out = {"node_tok": torch.full((b, M), 77, **i32), "node_parent": torch.full((b, M), 77, **i32),
           "node_depth": torch.full((b, M), 77, **i32), "n_nodes": torch.full((b,), 77, **i32),
           "cand_node": torch.full((b, Bc, n), 77, **i32),
           "mask": torch.full((b, M, M), 9, dtype=torch.uint8, device="cuda") if with_mask else None}
    B.spec_tree_metadata(cand, out["node_tok"], out["node_parent"], out["node_depth"], out["n_nodes"],
                         out["cand_node"], out["mask"])
    torch.cuda.synchronize()
    return out


META_CASES = [(1, 1, 1, 5), (3, 8, 3, 3), (2, 16, 4, 2), (1, 5, 7, 2), (4, 1, 5, 10), (2, 64, 3, 4), (1, 512, 8, 2)]


@pytest.mark.parametrize("b,Bc,n,V", META_CASES)
def test_tree_metadata_random_candidates(b, Bc, n, V):
    rng = np.random.default_rng(b * 100 + Bc)
    cand = rng.integers(0, V, (b, Bc, n)).astype(np.int32)
    log("tree metadata b=%d B=%d n=%d V=%d" % (b, Bc, n, V))
    want = O.tree_metadata(cand)
    got = _device_metadata(torch.from_numpy(cand).cuda())
    for key, w in want.items():
        assert np.array_equal(got[key].cpu().numpy(), w), key


def test_tree_metadata_of_a_real_draft_and_without_mask():
    wl = W.Workload("meta", 128, 128, 700, 3, (4, 3, 2), 12, 3, "bf16", "f32", 0.6, seed=2, emb_std=0.3)
    gen = W.make_generator(wl.seed, "cuda")
    w = W.make_speculator(wl, gen, device="cuda")
    state, last = W.make_draft_inputs(wl, gen, device="cuda")
    step = Step(wl, w)
    step.draft(state, last)
    got = _device_metadata(step.cand_tokens, with_mask=False)
    want = O.tree_metadata(step.cand_tokens.cpu().numpy())
    for key in ("node_tok", "node_parent", "node_depth", "n_nodes", "cand_node"):
        assert np.array_equal(got[key].cpu().numpy(), want[key]), key
    # candidates of a pruned (4, 3, 2) tree share prefixes: fewer nodes than B * n
    assert (want["n_nodes"] < wl.B * wl.n_predict).all() and (want["n_nodes"] >= wl.n_predict).all()


def test_tree_metadata_rejects_bad_arguments():
    i32 = dict(dtype=torch.int32, device="cuda")
    big = torch.zeros((1, 1024, 8), **i32)                  # B * n > 4096: rejected by the library
    o = torch.zeros((1, 8192), **i32)
    with pytest.raises(B.SpecError):
        B.spec_tree_metadata(big, o, o, o, torch.zeros((1,), **i32), torch.zeros((1, 1024, 8), **i32))
    nine = torch.zeros((1, 2, 9), **i32)                    # n_predict > 8
    o18 = torch.zeros((1, 18), **i32)
    with pytest.raises(B.SpecError):
        B.spec_tree_metadata(nine, o18, o18, o18, torch.zeros((1,), **i32), torch.zeros((1, 2, 9), **i32))
    with pytest.raises(ValueError):                         # an output of the wrong size never reaches the library
        B.spec_tree_metadata(torch.zeros((1, 2, 3), **i32), o, o, o, torch.zeros((1,), **i32),
                             torch.zeros((1, 2, 3), **i32))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_advance_matches_oracle(dtype):
    g = torch.Generator().manual_seed(5)
    b, Bc, n, E = 5, 6, 4, 136 if dtype == torch.float32 else 129   # 129 bf16 = 258 bytes: the unaligned path
    hidden = torch.randn((b, Bc, n + 1, E), generator=g).to(dtype)
    best = torch.randint(0, Bc, (b,), generator=g, dtype=torch.int32)
    acc = torch.randint(0, n + 1, (b,), generator=g, dtype=torch.int32)
    out = torch.randint(0, 1000, (b, n + 1), generator=g, dtype=torch.int32)
    ns = torch.zeros((b, E), dtype=dtype, device="cuda")
    nt = torch.zeros((b,), dtype=torch.int32, device="cuda")
    B.spec_advance(hidden.cuda(), best.cuda(), acc.cuda(), out.cuda(), ns, nt)
    torch.cuda.synchronize()
    ws, wt = O.advance(hidden.float().numpy(), best.numpy(), acc.numpy(), out.numpy())
    assert np.array_equal(ns.float().cpu().numpy(), ws.astype(np.float32))
    assert np.array_equal(nt.cpu().numpy(), wt)


def test_three_steps_chained_on_the_device_match_an_oracle_loop():
    """draft -> verify -> advance -> draft ... enqueued on one stream with no host read in
    between; the base model is played by pre-generated logits and hidden states per step."""
    wl = W.Workload("loop", 256, 256, 900, 3, (3, 2, 2), 6, 4, "bf16", "f32", 0.6, seed=8, emb_std=0.3)
    gen = W.make_generator(wl.seed, "cpu")
    w = W.make_speculator(wl, gen, device="cpu", ln_affine="random")
    state0, last0 = W.make_draft_inputs(wl, gen, device="cpu")
    steps = 3
    b, Bc, n, E, V = wl.batch, wl.B, wl.n_predict, wl.emb_dim, wl.vocab
    logits = [torch.randn((b, Bc, n + 1, V), generator=gen) for _ in range(steps)]
    hidden = [torch.randn((b, Bc, n + 1, E), generator=gen).to(torch.bfloat16) for _ in range(steps)]
    # favour acceptance a little: boost a fixed token so that candidates containing it match sometimes
    for lg in logits:
        lg[..., 7] += 1.5

    # ---- device: everything enqueued, one synchronisation at the end
    wd = {k: [t.cuda() for t in v] for k, v in w.items()}
    st = [Step(wl, wd, debug=True) for _ in range(steps)]   # one set of output tensors per step (kept for the check)
    state = state0.cuda()
    last = last0.cuda()
    states, lasts = [], []
    for s in range(steps):
        st[s].draft(state, last)
        st[s].verify(logits[s].cuda())
        nstate = torch.empty((b, E), dtype=torch.bfloat16, device="cuda")
        ntok = torch.empty((b,), dtype=torch.int32, device="cuda")
        B.spec_advance(hidden[s].cuda(), st[s].best_cand, st[s].accept_len, st[s].out_tokens, nstate, ntok)
        states.append(nstate)
        lasts.append(ntok)
        state, last = nstate, ntok
    torch.cuda.synchronize()

    # ---- oracle loop on the host, following the device wherever a near-tie lets them differ
    wn = W.weights_to_numpy(w)
    o_state, o_last = W.to_numpy_f32(state0), last0.numpy()
    for s in range(steps):
        od = O.draft(wn, o_state, o_last, wl.top_k, wl.B, state_dtype="bf16", keep_logits=True)
        dev_cand = st[s].cand_tokens.cpu().numpy()

        def along(q, path, o_state=o_state, o_last=o_last):
            return O.logp_along_path(wn, o_state[q], int(o_last[q]), path, wl.n_predict, state_dtype="bf16")

        # the same tie-aware rule as the single-step tests: a differing choice must be valid inside the
        # 1e-3 band on the oracle's head evaluated on the device's own state rows
        rep = parity.compare_draft(od, tables_to_numpy(st[s]),
                                   {"tokens": dev_cand, "scores": st[s].cand_scores.cpu().numpy(),
                                    "leaf": st[s].cand_leaf.cpu().numpy()}, wl.top_k, wn["head"], along_path=along)
        log("step %d: %s" % (s, rep.line()))
        assert rep.rows_checked + rep.rows_skipped_below_exempt == sum(wl.rows())
        assert rep.rows_exempt <= 1
        ov = O.verify(logits[s].numpy(), dev_cand)          # verify on the device's candidates: exact
        assert np.array_equal(ov.accept_len, st[s].accept_len.cpu().numpy())
        assert np.array_equal(ov.best_cand, st[s].best_cand.cpu().numpy())
        assert np.array_equal(ov.out_tokens, st[s].out_tokens.cpu().numpy())
        ns, nt = O.advance(hidden[s].float().numpy(), ov.best_cand, ov.accept_len, ov.out_tokens)
        assert np.array_equal(states[s].float().cpu().numpy(), ns.astype(np.float32))
        assert np.array_equal(lasts[s].cpu().numpy(), nt)
        o_state, o_last = ns, nt
