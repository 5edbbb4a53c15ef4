"""CPU-side checks of the boundary: the library loads, exports every symbol the
header declares, and rejects bad arguments before any HIP call (so these run
without a GPU)."""
import ctypes as C
import os
import re

import pytest

from paper_2404_19124_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    with open(os.path.join(ROOT, "include", "spec.h")) as f:
        text = f.read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spec_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert set(names) == set(B.EXPORTS), names
    lib = B.lib()
    for name in names:
        assert getattr(lib, name) is not None


def test_header_constants_match_binding():
    with open(os.path.join(ROOT, "include", "spec.h")) as f:
        text = f.read()
    for name in ("SPEC_MAX_STAGES", "SPEC_MAX_TOPK", "SPEC_MAX_LEAVES"):
        assert int(re.search(r"#define\s+%s\s+(\d+)" % name, text).group(1)) == getattr(B, name)
    assert C.sizeof(B.spec_config_t) == 4 * 9 + 4 * B.SPEC_MAX_STAGES


def test_version_and_last_error():
    assert B.spec_version() == (0, 1)
    assert isinstance(B.spec_last_error(), str)


def _create(cfg):
    n = max(1, min(cfg.n_predict, B.SPEC_MAX_STAGES))
    fake = (C.c_void_p * n)(*([0x1000] * n))     # never dereferenced: validation fails first
    w = B.spec_weights_t(*[C.cast(fake, C.POINTER(C.c_void_p))] * 5)
    h = C.c_void_p()
    return B.lib().spec_create(C.byref(cfg), C.byref(w), None, C.byref(h)), h


@pytest.mark.parametrize("kw,status", [
    (dict(n_predict=0), B.SPEC_EINVAL),
    (dict(n_predict=9), B.SPEC_EINVAL),
    (dict(vocab=0), B.SPEC_EINVAL),
    (dict(weight_dtype=7), B.SPEC_EDTYPE),
    (dict(emb_dim=100), B.SPEC_ESHAPE),                 # bf16 needs multiples of 64
    (dict(weight_dtype="f32", inner_dim=20), B.SPEC_ESHAPE),
    (dict(max_batch=0), B.SPEC_EINVAL),
    (dict(max_top_k=(0, 1, 1)), B.SPEC_EINVAL),
    (dict(max_top_k=(9, 1, 1)), B.SPEC_EINVAL),
    (dict(max_top_k=(8, 8, 8), n_predict=3, vocab=4), B.SPEC_EINVAL),      # k > V
    (dict(n_predict=5, max_top_k=(8, 8, 8, 8, 8)), B.SPEC_ESHAPE),         # too many leaves
])
def test_create_rejects_bad_config_before_touching_the_device(kw, status):
    base = dict(n_predict=3, emb_dim=128, inner_dim=128, vocab=1000, weight_dtype="bf16", max_batch=2,
                max_top_k=(4, 3, 2))
    base.update(kw)
    cfg = B.make_config(**base)
    got, h = _create(cfg)
    assert got == status, B.spec_last_error()
    assert not h.value
    assert B.spec_last_error()


def test_create_rejects_null_pointers():
    cfg = B.make_config(3, 128, 128, 1000, "bf16", 2, (4, 3, 2))
    h = C.c_void_p()
    assert B.lib().spec_create(C.byref(cfg), None, None, C.byref(h)) == B.SPEC_EINVAL
    assert B.lib().spec_create(None, None, None, C.byref(h)) == B.SPEC_EINVAL
    null = (C.c_void_p * 3)(0, 0, 0)
    w = B.spec_weights_t(*[C.cast(null, C.POINTER(C.c_void_p))] * 5)
    assert B.lib().spec_create(C.byref(cfg), C.byref(w), None, C.byref(h)) == B.SPEC_EINVAL
    assert "stage 0" in B.spec_last_error()


def test_draft_and_verify_reject_bad_arguments_without_a_device():
    lib = B.lib()
    assert lib.spec_draft(None, None, None, 1, None, 1, None, None, None, None, None) == B.SPEC_EINVAL
    p = C.c_void_p(0x1000)
    # verify: nulls, dtype, ranges
    assert lib.spec_verify(None, 0, p, 1, 1, 1, 10, p, p, p, p, p, None, None) == B.SPEC_EINVAL
    assert lib.spec_verify(p, 5, p, 1, 1, 1, 10, p, p, p, p, p, None, None) == B.SPEC_EDTYPE
    assert lib.spec_verify(p, 0, p, 0, 1, 1, 10, p, p, p, p, p, None, None) == B.SPEC_EINVAL
    assert lib.spec_verify(p, 0, p, 1, 1, 0, 10, p, p, p, p, p, None, None) == B.SPEC_EINVAL
    assert lib.spec_verify(p, 0, p, 1, 1, 9, 10, p, p, p, p, p, None, None) == B.SPEC_EINVAL
    assert lib.spec_verify(p, 0, p, 1 << 20, 1 << 10, 3, 10, p, p, p, p, p, None, None) == B.SPEC_ESHAPE
    assert lib.spec_head_logp(None, 0, p, 1, p, None) == B.SPEC_EINVAL
    assert lib.spec_model_scalars(None, None, None, None) == B.SPEC_EINVAL
    lib.spec_destroy(None)      # allowed


def test_binding_validates_tensors_on_the_host_before_any_pointer_crosses_the_boundary(monkeypatch):
    """Element type, shape, strides and device of every tensor argument are checked in the binding
    (the library only sees raw addresses).  No GPU needed: the checks run before the library call."""
    import types

    import torch
    cfg = B.make_config(3, 128, 64, 1000, "bf16", 4, (4, 3, 2))
    model = types.SimpleNamespace(cfg=cfg, handle=None)
    i32 = torch.int32
    state = torch.zeros((2, 128), dtype=torch.bfloat16)
    last = torch.zeros((2,), dtype=i32)
    ct, cs, cl = torch.zeros((2, 6, 3), dtype=i32), torch.zeros((2, 6)), torch.zeros((2, 6), dtype=i32)

    def draft(**kw):
        a = dict(state=state, last_tok=last, top_k=(4, 3, 2), B=6, cand_tokens=ct, cand_scores=cs, cand_leaf=cl)
        a.update(kw)
        return B.spec_draft(model, a["state"], a["last_tok"], a["top_k"], a["B"], a["cand_tokens"], a["cand_scores"],
                            a["cand_leaf"], a.get("dbg"))

    with pytest.raises(ValueError, match="device tensor"):      # everything right except the device
        draft()
    logits = torch.zeros((2, 6, 4, 50))
    outs = dict(greedy=torch.zeros((2, 6, 4), dtype=i32), accept_len=torch.zeros((2,), dtype=i32),
                best_cand=torch.zeros((2,), dtype=i32), out_tokens=torch.zeros((2, 4), dtype=i32),
                n_out=torch.zeros((2,), dtype=i32))
    with pytest.raises(ValueError, match="device tensor"):
        B.spec_verify(logits, ct, **outs)
    monkeypatch.setattr(B, "_CHECK_DEVICE", False)              # the remaining checks, on host tensors
    with pytest.raises(ValueError, match="top_k needs 3"):
        draft(top_k=(4, 3))
    with pytest.raises(ValueError, match="last_tok must have dtype torch.int32"):
        draft(last_tok=last.long())                             # torch.randint's default type
    with pytest.raises(ValueError, match="state must have dtype torch.bfloat16"):
        draft(state=state.float())
    with pytest.raises(ValueError, match="state must have shape"):
        draft(state=torch.zeros((2, 64), dtype=torch.bfloat16))
    with pytest.raises(ValueError, match="cand_tokens must have shape"):
        draft(cand_tokens=torch.zeros((2, 5, 3), dtype=i32))
    with pytest.raises(ValueError, match="cand_scores must be contiguous"):
        draft(cand_scores=torch.zeros((6, 2)).t())
    with pytest.raises(ValueError, match="stage_state"):
        draft(dbg={"stage_state": torch.zeros((3, 64), dtype=torch.bfloat16)})   # needs 2 + 8 + 24 rows

    with pytest.raises(ValueError, match="float32 or bfloat16"):
        B.spec_verify(logits.half(), ct, **outs)
    with pytest.raises(ValueError, match="cand_tokens must have shape"):
        B.spec_verify(logits, ct[:, :5], **outs)
    with pytest.raises(ValueError, match="greedy must have shape"):
        B.spec_verify(logits, ct, **dict(outs, greedy=torch.zeros((2, 6, 3), dtype=i32)))
    with pytest.raises(ValueError, match="next_state"):
        B.spec_advance(torch.zeros((2, 6, 4, 128)), outs["best_cand"], outs["accept_len"], outs["out_tokens"],
                       torch.zeros((2, 64)), torch.zeros((2,), dtype=i32))
    with pytest.raises(ValueError, match="logp must have shape"):
        B.spec_head_logp(model, 0, torch.zeros((5, 64), dtype=torch.bfloat16), torch.zeros((5, 999)))
    with pytest.raises(ValueError, match="weights"):
        B.SpecModel(cfg, {k: [torch.zeros(1)] * 3 for k in ("proj", "emb", "head", "ln_gamma", "ln_beta")})


def test_create_rejects_weights_that_are_not_16_byte_aligned():
    cfg = B.make_config(3, 128, 128, 1000, "bf16", 2, (4, 3, 2))
    odd = (C.c_void_p * 3)(0x1008, 0x1000, 0x1000)
    ok = (C.c_void_p * 3)(0x1000, 0x1000, 0x1000)
    for bad_field in range(5):
        ptrs = [C.cast(odd if f == bad_field else ok, C.POINTER(C.c_void_p)) for f in range(5)]
        h = C.c_void_p()
        assert B.lib().spec_create(C.byref(cfg), C.byref(B.spec_weights_t(*ptrs)), None, C.byref(h)) == B.SPEC_EINVAL
        assert "16-byte aligned" in B.spec_last_error() and not h.value


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        B.lib()
