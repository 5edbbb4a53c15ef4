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


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        B.lib()
