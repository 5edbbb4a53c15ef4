"""spec_draft_static (the draft whose workspace lives in the library's static device array, for
callers that cannot allocate) against spec_draft, through the C ABI: identical kernels on
identical inputs, so every output must be bit-identical.  Two calls in a row, the second with a
smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

from paper_2404_19124_amd import binding as B
from paper_2404_19124_amd import workloads as W
from paper_2404_19124_amd.runner import Step
from tests.gpu_common import log

pytestmark = pytest.mark.gpu


def _outputs(batch, Bc, n):
    i32 = dict(dtype=torch.int32, device="cuda")
    return (torch.full((batch, Bc, n), -7, **i32), torch.full((batch, Bc), -7.0, device="cuda"),
            torch.full((batch, Bc), -7, **i32))


def _both(step, state, last, top_k, Bc):
    """(outputs of spec_draft, outputs of spec_draft_static) for one input."""
    n = step.wl.n_predict
    ref, got = _outputs(state.shape[0], Bc, n), _outputs(state.shape[0], Bc, n)
    B.spec_draft(step.model, state, last, top_k, Bc, *ref)
    torch.cuda.synchronize()
    B.spec_draft_static(step.model, state, last, top_k, Bc, *got)
    torch.cuda.synchronize()
    return ref, got


CASES = [
    # name, E, D, V, n, top_k, B, batch, dtype; second call: (batch2, top_k2, B2)
    ("skinny_d512", 512, 512, 1000, 3, (5, 3, 2), 10, 1, "bf16", (1, (2, 3, 1), 4)),
    ("skinny_b3", 128, 192, 1000, 3, (4, 3, 1), 9, 3, "bf16", (2, (2, 2, 1), 3)),
    ("dense_b7", 256, 128, 2049, 3, (5, 3, 2), 16, 7, "bf16", (3, (5, 2, 2), 7)),
    ("dense_b40_long_e", 1024, 128, 300, 2, (3, 2), 6, 40, "bf16", (17, (3, 1), 2)),
    ("f32_b5", 100, 72, 333, 3, (3, 3, 2), 7, 5, "f32", (2, (2, 3, 2), 12)),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_static_workspace_draft_equals_spec_draft_on_two_calls_in_a_row(case):
    name, E, D, V, n, top_k, Bc, batch, dtype, (batch2, top_k2, B2) = case
    wl = W.Workload(name, E, D, V, n, top_k, Bc, batch, dtype, "f32", 0.6, seed=31, emb_std=0.3)
    log("static draft %s" % name)
    gen = W.make_generator(wl.seed)
    w = {k: [t.cuda() for t in v] for k, v in W.make_speculator(wl, gen, ln_affine="random").items()}
    state, last = W.make_draft_inputs(wl, gen)
    state, last = state.cuda(), last.cuda()
    step = Step(wl, w)
    ref, got = _both(step, state, last, top_k, Bc)
    for a, b, what in zip(ref, got, ("cand_tokens", "cand_scores", "cand_leaf")):
        assert torch.equal(a, b), "first call: %s differs" % what
    assert int(got[2].min()) >= 0
    # second call, smaller: fewer sequences (other ones), a narrower tree
    state2, last2 = state[batch - batch2:].contiguous(), last[batch - batch2:].contiguous()
    ref2, got2 = _both(step, state2, last2, top_k2, B2)
    for a, b, what in zip(ref2, got2, ("cand_tokens", "cand_scores", "cand_leaf")):
        assert torch.equal(a, b), "second (smaller) call: %s differs" % what
    # and the first input once more: nothing of the smaller call is left behind
    ref3, got3 = _both(step, state, last, top_k, Bc)
    for a, b in zip(ref, got3):
        assert torch.equal(a, b)
    step.close()


def test_static_workspace_draft_at_the_7b_shape_and_its_size_limit():
    wl = W.WORKLOADS["llama7b_b1"]
    gen = W.make_generator(wl.seed, "cuda")
    w = W.make_speculator(wl, gen, device="cuda")
    state, last = W.make_draft_inputs(wl, gen, device="cuda")
    step = Step(wl, w, max_batch=64)
    ref, got = _both(step, state, last, wl.top_k, wl.B)
    for a, b in zip(ref, got):
        assert torch.equal(a, b)
    ref2, got2 = _both(step, state, last, (2, 1, 1), 2)
    for a, b in zip(ref2, got2):
        assert torch.equal(a, b)
    # 64 sequences of this model need more than the array holds: refused, nothing enqueued, model still fine
    s64 = state.expand(64, -1).contiguous()
    l64 = last.expand(64).contiguous()
    out = _outputs(64, wl.B, wl.n_predict)
    with pytest.raises(B.SpecError) as e:
        B.spec_draft_static(step.model, s64, l64, wl.top_k, wl.B, *out)
    assert e.value.status == B.SPEC_ESHAPE and "static array" in str(e.value)
    assert int(out[0].max()) == -7
    B.spec_draft(step.model, s64, l64, wl.top_k, wl.B, *out)      # the allocating entry point takes it
    torch.cuda.synchronize()
    assert torch.equal(out[0][0], ref[0][0]) and torch.equal(out[0][63], ref[0][0])
    step.close()


def test_static_workspace_draft_rejects_bad_arguments_like_spec_draft():
    wl = W.Workload("err", 64, 64, 100, 2, (2, 2), 4, 2, "bf16", "f32", 0.5)
    gen = W.make_generator(0)
    w = {k: [t.cuda() for t in v] for k, v in W.make_speculator(wl, gen).items()}
    step = Step(wl, w)
    state, last = W.make_draft_inputs(wl, gen)
    out = _outputs(2, 5, 2)
    with pytest.raises(B.SpecError) as e:
        B.spec_draft_static(step.model, state.cuda(), last.cuda(), wl.top_k, 5, *out)   # more candidates than leaves
    assert e.value.status == B.SPEC_EINVAL
    out = _outputs(2, 4, 2)
    with pytest.raises(B.SpecError) as e:
        B.spec_draft_static(step.model, state.cuda(), last.cuda(), (3, 2), 4, *out)     # above max_top_k
    assert e.value.status == B.SPEC_ESHAPE
    step.close()
