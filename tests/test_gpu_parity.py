"""GPU parity tests: the HIP path, called through the C ABI, against the CPU
oracle on identical seeded inputs.  Small shapes are compared element by element
(several tiles plus ragged tails); the full-size configurations are compared at
the launch configuration the benchmark times, on all sequences where the oracle
finishes in seconds and on sampled sequences otherwise."""
import os

import numpy as np
import pytest
import torch

from oracle import spec_oracle as O
from paper_2404_19124_amd import binding as B
from paper_2404_19124_amd import workloads as W
from paper_2404_19124_amd.runner import Step
from tests.gpu_common import compare_verify, log, run_workload

pytestmark = pytest.mark.gpu


def test_native_library_is_loaded_and_shares_the_hip_runtime():
    B.lib()
    with open("/proc/self/maps") as f:
        maps = f.read()
    assert "libspecdraft.so" in maps
    hips = {line.split()[-1] for line in maps.splitlines() if "libamdhip64" in line}
    assert len(hips) == 1, "two HIP runtimes in one process: %s" % hips
    assert B.spec_version() == (0, 1)


def test_tiny_configuration_full_step_and_stored_result():
    wl = W.WORKLOADS["tiny_b1"]
    rep, step, od, ov = run_workload(wl, gen_device="cpu")
    assert rep.rows_exempt == 0 and rep.cand_exempt == 0
    # the same numbers as the file written from the oracle alone
    stored = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "tiny_b1_seed0.txt")) as f:
        for line in f:
            if not line.startswith("#") and "=" in line:
                k, v = line.split("=")
                stored[k.strip()] = v.split()
    assert step.cand_leaf.cpu().numpy()[0].tolist() == [int(x) for x in stored["cand_leaf"]]
    assert step.cand_tokens.cpu().numpy()[0].reshape(-1).tolist() == [int(x) for x in stored["cand_tokens"]]
    # verify on the stored recipe's logits (speculator, inputs, then logits from one generator)
    gen = W.make_generator(wl.seed)
    W.make_speculator(wl, gen)
    W.make_draft_inputs(wl, gen)
    logits = W.make_base_logits(wl, torch.from_numpy(od.cand_tokens), gen).cuda()
    step.verify(logits)          # chained on the device's own candidates
    torch.cuda.synchronize()
    assert step.out_tokens.cpu().numpy()[0].tolist() == [int(x) for x in stored["out_tokens"]]
    assert int(step.accept_len[0]) == int(stored["accept_len"][0])
    assert int(step.best_cand[0]) == int(stored["best_cand"][0])
    assert step.accept_all.cpu().numpy()[0].tolist() == [int(x) for x in stored["accept_all"]]
    compare_verify(step, O.verify(W.to_numpy_f32(logits), od.cand_tokens), [0], wl.n_predict)


SMALL_BF16 = [
    # name, E, D, V, n, top_k, B, batch : rows per stage
    ("bf16_b1", 128, 192, 1000, 3, (4, 3, 2), 24, 1),       # 1, 4, 12      one-CU-per-tile path only
    ("bf16_b3", 128, 192, 1000, 3, (4, 3, 2), 10, 3),       # 3, 12, 36     both contraction paths
    ("bf16_b7", 256, 128, 2049, 3, (5, 3, 2), 16, 7),       # 7, 35, 105    ragged vocabulary, several row tiles
    ("bf16_b20_n2", 192, 256, 777, 2, (8, 8), 64, 20),      # 20, 160       widest top-k
    ("bf16_b2_n4", 64, 64, 300, 4, (3, 2, 2, 2), 24, 2),    # 2, 6, 12, 24  four stages
    ("bf16_chain_n7", 128, 128, 500, 7, (1,) * 7, 1, 2),    # k = 1 chain, 7 heads
    ("bf16_b1_n5", 128, 128, 500, 5, (2, 2, 1, 2, 1), 5, 1),
    ("bf16_b40_long_vocab", 64, 64, 33000, 2, (2, 2), 4, 40),  # 40, 80 rows: wide kernel with 64-row blocks
    # the same 64-row instance with per-lane lists of 4, 6 and 8 entries (top-k 4, 6, 8), 64 and 33 rows
    ("bf16_b40_long_vocab_k4", 64, 64, 33000, 2, (4, 1), 4, 40),
    ("bf16_b64_long_vocab_k6", 64, 64, 33000, 2, (6, 1), 6, 64),
    ("bf16_b33_long_vocab_k8", 64, 64, 33000, 2, (8, 1), 8, 33),
    # more than 64 rows with top-k 6 and 3: 96-row blocks with per-lane lists of 6 and of 3 entries
    ("bf16_b70_k6", 64, 128, 2049, 2, (6, 3), 8, 70),
    # 160-row state blocks of the wide kernel (chosen when 96-row blocks would need two tiles per range):
    # 5 K slabs = one steady group + tail, ragged vocabulary and rows; per-lane lists of 2 and of 4
    ("bf16_b31_tall_k2", 128, 320, 16500, 3, (5, 3, 2), 6, 31),   # 31, 155, 465
    ("bf16_b31_tall_k3", 128, 320, 16500, 3, (5, 3, 3), 6, 31),
    # 128-row state blocks (310 rows against 80 tiles: one tile per range with three blocks, two with four)
    ("bf16_b31_mid_k2", 128, 320, 20300, 3, (5, 2, 2), 6, 31),    # 31, 155, 310
    ("bf16_b31_mid_k3", 128, 320, 20300, 3, (5, 2, 3), 6, 31),
    # the same block heights with full 256-row tiles and two tiles per range (the cases above get short tiles)
    ("bf16_b31_mid_two_tiles", 64, 128, 36000, 3, (5, 2, 2), 6, 31),        # 310 rows, 141 tiles over 85 ranges
    ("bf16_b31_tall_two_tiles", 64, 128, 21400, 4, (5, 3, 2, 2), 6, 31),    # 930 rows, 84 tiles over 42 ranges
    # first projection split along K (long E, more than 16 rows): four parts, and two parts with two row blocks
    ("bf16_b20_long_e", 2048, 64, 300, 2, (2, 2), 4, 20),
    ("bf16_b40_long_e", 1024, 128, 300, 2, (3, 2), 6, 40),
    # a first projection of more than 64 rows: the wide kernel's store epilogue with four K parts
    ("bf16_b70_long_e", 2048, 64, 300, 2, (2, 2), 4, 70),
    # head and next projection launched apart (254 + 4 tiles against 256 ranges would make two ranges two tiles
    # long): the head alone, then the projection with two K parts on the wide kernel (155 rows)
    ("bf16_b31_proj_apart", 128, 1024, 65000, 3, (5, 2, 2), 6, 31),
    # the limits of the boundary: 4096 leaves with top-k 8 everywhere (rows 1, 8, 64, 512), eight stages,
    # a vocabulary smaller than one 16-row tile
    ("bf16_max_leaves", 64, 64, 300, 4, (8, 8, 8, 8), 64, 1),
    ("bf16_eight_stages", 64, 64, 200, 8, (2, 1, 2, 1, 2, 1, 2, 1), 16, 2),
    ("bf16_vocab_9", 64, 64, 9, 2, (8, 3), 24, 3),
]


@pytest.mark.parametrize("case", SMALL_BF16, ids=[c[0] for c in SMALL_BF16])
def test_small_bf16_shapes(case):
    name, E, D, V, n, top_k, Bc, batch = case
    wl = W.Workload(name, E, D, V, n, top_k, Bc, batch, "bf16", "f32", 0.6, seed=11, emb_std=0.3)
    if name == "bf16_b31_proj_apart":   # the case does take the path it is meant for
        assert B.spec_plan_contraction(155, D, V, 2, D)["proj_apart"] == 1
        assert B.spec_plan_contraction(155, D, 0, 0, D)["k_split"] == 2
    if name == "bf16_b70_long_e":
        p = B.spec_plan_contraction(70, E, 0, 0, D)
        assert p["kernel"] >= 1000 and p["k_split"] == 4
    rep, step, od, ov = run_workload(wl, ln_affine="random", gen_device="cpu")
    assert rep.rows_checked + rep.rows_skipped_below_exempt == sum(wl.rows())
    assert rep.rows_exempt <= max(1, sum(wl.rows()) // 100)


# Every stage at most 16 rows: the streaming kernel for every contraction - widths with one and two chunks
# per thread in the stage kernel, every merge width, several sequences, a 7-stage chain; with one or two
# sequences and no debug outputs the first stage is computed inside the first head's launch.
STREAMING_BF16 = [
    ("stream_d512_rows_1_5_15", 512, 512, 1000, 3, (5, 3, 2), 10, 1),    # the paper's tree shape, ragged vocabulary
    ("stream_d1024_b2", 1024, 1024, 2049, 3, (2, 2, 2), 8, 2),           # two sequences: 2, 4, 8 rows
    ("stream_d2048_k8", 2048, 2048, 777, 2, (8, 8), 64, 2),              # 16 rows, widest top-k: group merges
    ("stream_d512_chain_n7", 512, 512, 500, 7, (1,) * 7, 1, 2),          # k = 1 chain
    ("stream_d3072_b1", 3072, 3072, 640, 2, (6, 2), 12, 1),              # two chunks per thread, merge width 6
    ("stream_d1536_b1", 512, 1536, 700, 2, (8, 2), 16, 1),               # E != D, 192 chunks per row
    ("stream_d4096_b2_chain", 512, 4096, 300, 4, (1,) * 4, 1, 2),        # the 7B width
    ("stream_d512_b3", 512, 512, 1000, 3, (3, 2, 1), 6, 3),              # 3, 9, 18 rows: the last stage takes the dense kernel
    ("stream_d4096_rows_16", 4096, 4096, 300, 3, (4, 4, 1), 16, 1),      # 16 rows: four rounds in two passes
    ("stream_d256_b16", 128, 256, 500, 2, (1, 1), 1, 16),                # 16 sequences: the tree step loops over them
]


@pytest.mark.parametrize("case", STREAMING_BF16, ids=[c[0] for c in STREAMING_BF16])
def test_streaming_kernel_shapes(case):
    name, E, D, V, n, top_k, Bc, batch = case
    wl = W.Workload(name, E, D, V, n, top_k, Bc, batch, "bf16", "f32", 0.6, seed=17, emb_std=0.3)
    rep, step, od, ov = run_workload(wl, ln_affine="random", gen_device="cpu")
    assert rep.rows_checked + rep.rows_skipped_below_exempt == sum(wl.rows())
    assert rep.rows_exempt <= 1
    # repeated calls on the same model
    gen = W.make_generator(wl.seed, "cpu")
    W.make_speculator(wl, gen, device="cpu", ln_affine="random")
    state, last = W.make_draft_inputs(wl, gen, device="cpu")
    want = step.cand_tokens.clone()
    for _ in range(3):
        step.cand_tokens.zero_()
        step.draft(state.cuda(), last.cuda())
    torch.cuda.synchronize()
    assert torch.equal(step.cand_tokens, want)


SMALL_F32 = [
    ("f32_b1", 256, 256, 1024, 3, (4, 3, 2), 24, 1),
    ("f32_b5", 100, 72, 333, 3, (3, 3, 2), 7, 5),           # nothing a multiple of the tile sizes
    ("f32_b2_n4", 48, 64, 97, 4, (2, 2, 2, 2), 16, 2),
]


@pytest.mark.parametrize("case", SMALL_F32, ids=[c[0] for c in SMALL_F32])
def test_small_f32_shapes(case):
    name, E, D, V, n, top_k, Bc, batch = case
    wl = W.Workload(name, E, D, V, n, top_k, Bc, batch, "f32", "f32", 0.6, seed=5, emb_std=0.3)
    rep, step, od, ov = run_workload(wl, ln_affine="random", gen_device="cpu")
    assert rep.rows_exempt == 0
    assert rep.max_state_rel < 1e-4 and rep.max_logp_abs < 1e-3


def test_bf16_logits_and_bf16_ties_in_verify():
    wl = W.Workload("bf16_logits", 128, 128, 20000, 3, (4, 3, 2), 16, 3, "bf16", "bf16", 0.6, seed=3)
    rep, step, od, ov = run_workload(wl, gen_device="cpu")


VERIFY_CASES = [
    # b, B, n, V, dtype
    (1, 1, 1, 1, "f32"), (2, 3, 3, 5, "f32"), (3, 16, 3, 1023, "f32"), (2, 5, 4, 4099, "bf16"),
    (4, 32, 3, 32000, "f32"), (1, 64, 7, 1000, "bf16"), (5, 2, 2, 70001, "f32"),
]


@pytest.mark.parametrize("b,Bc,n,V,dtype", VERIFY_CASES)
def test_verify_shapes_and_edges(b, Bc, n, V, dtype):
    g = torch.Generator().manual_seed(b * 1000 + V)
    logits = torch.randn((b, Bc, n + 1, V), generator=g)
    cand = torch.randint(0, V, (b, Bc, n), generator=g, dtype=torch.int32)
    hit = torch.rand((b, Bc, n), generator=g) < 0.7
    boost = torch.zeros((b, Bc, n, 1))
    boost[hit.unsqueeze(-1)] = 20.0
    logits[:, :, :n, :].scatter_add_(3, cand.long().unsqueeze(-1), boost)
    if V > 8:                      # planted exact ties: the smaller index must win
        logits[0, 0, 0, 7] = 50.0
        logits[0, 0, 0, 3] = 50.0
    logits = logits.to(torch.bfloat16 if dtype == "bf16" else torch.float32)
    wl = W.Workload("v", 64, 64, V, n, (1,) * n, Bc, b, "f32", dtype, 0.5)
    step = _bare_step(wl)
    step.verify(logits.cuda(), cand.cuda())
    torch.cuda.synchronize()
    ov = O.verify(logits.float().numpy(), cand.numpy())
    compare_verify(step, ov, list(range(b)), n)
    if V > 8:
        assert int(step.greedy[0, 0, 0]) == 3


class _bare_step(Step):
    """Outputs of a step without a model (spec_verify needs none)."""

    def __init__(self, wl):
        self.wl = wl
        dev = "cuda"
        b, n, Bc = wl.batch, wl.n_predict, wl.B
        i32 = dict(dtype=torch.int32, device=dev)
        self.cand_tokens = torch.empty((b, Bc, n), **i32)
        self.greedy = torch.empty((b, Bc, n + 1), **i32)
        self.accept_len = torch.empty((b,), **i32)
        self.best_cand = torch.empty((b,), **i32)
        self.out_tokens = torch.empty((b, n + 1), **i32)
        self.n_out = torch.empty((b,), **i32)
        self.accept_all = torch.empty((b, Bc), **i32)


def test_verify_unaligned_rows_take_the_scalar_path():
    # V * 4 bytes not a multiple of 16 and a base pointer off by one element
    b, Bc, n, V = 2, 3, 2, 1001
    g = torch.Generator().manual_seed(9)
    buf = torch.randn(b * Bc * (n + 1) * V + 1, generator=g).cuda()
    logits = buf[1:].view(b, Bc, n + 1, V)
    cand = torch.randint(0, V, (b, Bc, n), generator=g, dtype=torch.int32)
    wl = W.Workload("v", 64, 64, V, n, (1,) * n, Bc, b, "f32", "f32", 0.5)
    step = _bare_step(wl)
    step.verify(logits, cand.cuda())
    torch.cuda.synchronize()
    compare_verify(step, O.verify(logits.cpu().numpy(), cand.numpy()), list(range(b)), n)


def test_draft_is_deterministic_and_reusable():
    wl = W.Workload("det", 128, 192, 1000, 3, (4, 3, 2), 10, 3, "bf16", "f32", 0.6, seed=2, emb_std=0.3)
    gen = W.make_generator(2)
    w = {k: [t.cuda() for t in v] for k, v in W.make_speculator(wl, gen).items()}
    state, last = W.make_draft_inputs(wl, gen)
    step = Step(wl, w, debug=True)
    outs = []
    for _ in range(3):
        step.draft(state.cuda(), last.cuda())
        torch.cuda.synchronize()
        outs.append((step.cand_tokens.clone(), step.cand_scores.clone(), step.cand_leaf.clone(),
                     step.dbg["stage_state"].clone(), step.dbg["topk_logp"].clone()))
    for o in outs[1:]:
        for a, b in zip(outs[0], o):
            assert torch.equal(a, b)
    # a smaller call on the same model (fewer sequences, narrower tree) still matches the oracle
    wl2 = W.small_variant(wl, batch=1, top_k=(2, 3, 1), B=6)
    step2 = Step(wl2, w, debug=True, max_batch=3, max_top_k=(4, 3, 2))
    step2.draft(state[:1].cuda(), last[:1].cuda())
    torch.cuda.synchronize()
    od = O.draft(W.weights_to_numpy({k: [t.cpu() for t in v] for k, v in w.items()}), W.to_numpy_f32(state[:1]),
                 last[:1].numpy(), wl2.top_k, wl2.B, state_dtype="bf16")
    assert np.array_equal(step2.cand_tokens.cpu().numpy(), od.cand_tokens)
    assert np.array_equal(step2.cand_leaf.cpu().numpy(), od.cand_leaf)


@pytest.mark.parametrize("batch", [1, 24])
def test_draft_and_verify_replay_from_a_hip_graph(batch):
    """The step only enqueues kernels, so a caller may capture it in a HIP graph: every replay, with the
    program's own eager work and synchronisations in between, reproduces the eager step (batch 1: the
    streaming kernels; batch 24: the dense ones with the split first projection)."""
    wl = W.Workload("graph", 1024, 128, 2049, 3, (4, 3, 2), 10, batch, "bf16", "f32", 0.6, seed=9, emb_std=0.3)
    gen = W.make_generator(9)
    w = {k: [t.cuda() for t in v] for k, v in W.make_speculator(wl, gen).items()}
    step = Step(wl, w)
    inputs = []
    for _ in range(3):
        state, last = W.make_draft_inputs(wl, gen)
        logits = torch.randn((wl.batch, wl.B, wl.n_predict + 1, wl.vocab), generator=gen)
        inputs.append((state.cuda(), last.cuda(), logits.cuda()))
    outs = ("cand_tokens", "cand_scores", "cand_leaf", "greedy", "accept_len", "best_cand", "out_tokens", "n_out")
    eager = []
    for state, last, logits in inputs:
        step.draft(state, last)
        step.verify(logits)
        torch.cuda.synchronize()
        eager.append([getattr(step, name).clone() for name in outs])
    s_state, s_last, s_logits = (t.clone() for t in inputs[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):      # a warm-up on the capture stream, as torch asks for
        step.draft(s_state, s_last)
        step.verify(s_logits)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step.draft(s_state, s_last)
        step.verify(s_logits)
    for rep in range(2):
        for (state, last, logits), want in zip(inputs, eager):
            s_state.copy_(state)
            s_last.copy_(last)
            s_logits.copy_(logits)
            graph.replay()
            torch.cuda.synchronize()
            for name, ref in zip(outs, want):
                assert torch.equal(getattr(step, name), ref), (name, rep)
            # eager work of the program between the replays
            step.draft(inputs[rep][0], inputs[rep][1])
            torch.cuda.synchronize()
    step.close()


def test_no_token_conditioning_mode_and_tied_weights():
    wl = W.Workload("medusa", 128, 128, 600, 3, (3, 3, 2), 18, 2, "bf16", "f32", 0.6, seed=4, emb_std=0.3)
    rep, step, od, ov = run_workload(wl, w_s=1.0, w_e=0.0, gen_device="cpu")
    t = step.debug_tables()
    for i in range(3):
        per = wl.rows()[i] // wl.batch
        tok = t["tok"][i].view(wl.batch, per, -1)
        assert torch.equal(tok, tok[:, :1].expand_as(tok))       # same top-k under every parent
    wl = W.Workload("tied", 128, 128, 600, 4, (3, 2, 2, 2), 24, 2, "bf16", "f32", 0.6, seed=6, emb_std=0.3)
    run_workload(wl, tied=True, gen_device="cpu")


def test_head_logp_entry_point_matches_oracle():
    for dtype, rows in (("bf16", 5), ("bf16", 40), ("f32", 9)):
        wl = W.Workload("logp", 128, 128, 1234, 2, (3, 2), 6, 14, dtype, "f32", 0.6, seed=8)
        gen = W.make_generator(8)
        w = W.make_speculator(wl, gen)
        step = Step(wl, {k: [t.cuda() for t in v] for k, v in w.items()})
        s = torch.randn(rows, wl.inner_dim, generator=gen).to(torch.bfloat16 if dtype == "bf16" else torch.float32)
        out = torch.empty((rows, wl.vocab), dtype=torch.float32, device="cuda")
        B.spec_head_logp(step.model, 1, s.cuda(), out)
        torch.cuda.synchronize()
        want, _ = O.log_softmax(O.head_logits(s.float().numpy(), W.to_numpy_f32(w["head"][1])))
        got = out.cpu().numpy().astype(np.float64)
        assert np.abs(got - want).max() < (2e-3 if dtype == "bf16" else 1e-4)
        assert np.allclose(np.exp(got).sum(-1), 1.0, atol=1e-4)


@pytest.mark.parametrize("rows,V", [(48, 33000), (120, 33000), (300, 20300), (465, 16500)])
def test_head_logp_through_the_wide_kernels_store_epilogue(rows, V):
    """Full log-softmax rows through the wide dense kernel's store epilogue for the head matrix: 64-row
    blocks with short tiles, 96-row blocks with short tiles, 128- and 160-row blocks."""
    wl = W.Workload("logp_wide", 128, 320, V, 2, (3, 2), 6, 160, "bf16", "f32", 0.6, seed=12)
    gen = W.make_generator(12)
    w = W.make_speculator(wl, gen)
    step = Step(wl, {k: [t.cuda() for t in v] for k, v in w.items()})
    s = torch.randn(rows, wl.inner_dim, generator=gen).to(torch.bfloat16)
    out = torch.empty((rows, wl.vocab), dtype=torch.float32, device="cuda")
    B.spec_head_logp(step.model, 0, s.cuda(), out)
    torch.cuda.synchronize()
    want, _ = O.log_softmax(O.head_logits(s.float().numpy(), W.to_numpy_f32(w["head"][0])))
    got = out.cpu().numpy().astype(np.float64)
    assert np.abs(got - want).max() < 2e-3
    assert np.allclose(np.exp(got).sum(-1), 1.0, atol=1e-4)
    step.close()


def test_runtime_argument_errors():
    wl = W.Workload("err", 64, 64, 100, 2, (2, 2), 4, 2, "bf16", "f32", 0.5)
    gen = W.make_generator(0)
    w = {k: [t.cuda() for t in v] for k, v in W.make_speculator(wl, gen).items()}
    step = Step(wl, w)
    state, last = W.make_draft_inputs(wl, gen)
    i32 = dict(dtype=torch.int32, device="cuda")
    st3 = torch.zeros((3, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.SpecError) as e:        # batch above max_batch
        B.spec_draft(step.model, st3, torch.zeros(3, **i32), wl.top_k, wl.B, torch.zeros((3, wl.B, 2), **i32),
                     torch.zeros((3, wl.B), device="cuda"), torch.zeros((3, wl.B), **i32))
    assert e.value.status == B.SPEC_ESHAPE
    with pytest.raises(B.SpecError) as e:        # top_k above max_top_k
        B.spec_draft(step.model, state.cuda(), last.cuda(), (3, 2), wl.B, step.cand_tokens, step.cand_scores,
                     step.cand_leaf)
    assert e.value.status == B.SPEC_ESHAPE
    with pytest.raises(B.SpecError) as e:        # more candidates than leaves
        B.spec_draft(step.model, state.cuda(), last.cuda(), wl.top_k, 5, torch.zeros((2, 5, 2), **i32),
                     torch.zeros((2, 5), device="cuda"), torch.zeros((2, 5), **i32))
    assert e.value.status == B.SPEC_EINVAL
    # the binding refuses what the library could not check: element type, shape, strides
    with pytest.raises(ValueError):
        B.spec_draft(step.model, state.cuda(), last.cuda().long(), wl.top_k, wl.B, step.cand_tokens, step.cand_scores,
                     step.cand_leaf)
    with pytest.raises(ValueError):
        B.spec_draft(step.model, state.cuda(), last.cuda(), wl.top_k, wl.B, step.cand_tokens[:, :2], step.cand_scores,
                     step.cand_leaf)
    # a state that does not start on a 16-byte boundary (a view shifted by one bf16 element)
    shifted = torch.zeros(wl.batch * wl.emb_dim + 8, dtype=torch.bfloat16, device="cuda")[1:1 + wl.batch * wl.emb_dim]
    with pytest.raises(B.SpecError) as e:
        B.spec_draft(step.model, shifted.view(wl.batch, wl.emb_dim), last.cuda(), wl.top_k, wl.B, step.cand_tokens,
                     step.cand_scores, step.cand_leaf)
    assert e.value.status == B.SPEC_EINVAL
    # the model still works after rejected calls
    step.draft(state.cuda(), last.cuda())
    torch.cuda.synchronize()
    assert int(step.cand_leaf.min()) >= 0
