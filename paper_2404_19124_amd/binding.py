"""ctypes binding of libspecdraft.so: the same names as include/spec.h, argument
marshalling only.  Every step of the path runs in the library's kernels; torch
is used for device memory and the current stream, nothing else.

The library is built in-tree by `python -m paper_2404_19124_amd.build`.  If it
is missing this module raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import torch  # imported before the library is loaded so both share one HIP runtime

SPEC_MAX_STAGES = 8
SPEC_MAX_TOPK = 8
SPEC_MAX_LEAVES = 4096
SPEC_F32, SPEC_BF16 = 0, 1
SPEC_OK, SPEC_EINVAL, SPEC_ESHAPE, SPEC_EDTYPE, SPEC_ENOMEM, SPEC_EHIP = 0, -1, -2, -3, -4, -5

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libspecdraft.so")

EXPORTS = ["spec_create", "spec_destroy", "spec_draft", "spec_verify", "spec_head_logp", "spec_model_scalars",
           "spec_profile_enable", "spec_profile_read", "spec_copy_probe", "spec_set_fused", "spec_fused_timeout", "spec_fused_phase_us", "spec_tree_metadata", "spec_advance", "spec_plan_contraction", "spec_last_error", "spec_version"]


class SpecError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("libspecdraft status %d: %s" % (status, message))
        self.status = status


class spec_config_t(C.Structure):
    _fields_ = [("n_predict", C.c_int32), ("emb_dim", C.c_int32), ("inner_dim", C.c_int32), ("vocab", C.c_int32),
                ("weight_dtype", C.c_int32), ("state_weight", C.c_float), ("emb_weight", C.c_float),
                ("ln_eps", C.c_float), ("max_batch", C.c_int32), ("max_top_k", C.c_int32 * SPEC_MAX_STAGES)]


class spec_weights_t(C.Structure):
    _fields_ = [("proj", C.POINTER(C.c_void_p)), ("emb", C.POINTER(C.c_void_p)), ("head", C.POINTER(C.c_void_p)),
                ("ln_gamma", C.POINTER(C.c_void_p)), ("ln_beta", C.POINTER(C.c_void_p))]


class spec_plan_t(C.Structure):
    _fields_ = [(name, C.c_int32) for name in ("kernel", "block_rows", "tile_rows", "row_blocks", "ranges", "tiles",
                                               "parts", "k_split", "workgroups", "lds_bytes")]


class spec_debug_t(C.Structure):
    _fields_ = [("stage_state", C.c_void_p), ("topk_tok", C.c_void_p), ("topk_logp", C.c_void_p),
                ("row_lse", C.c_void_p)]


class spec_launch_record_t(C.Structure):
    _fields_ = [("kernel", C.c_int32), ("rows", C.c_int32), ("weight_rows", C.c_int32), ("k", C.c_int32),
                ("ms", C.c_float)]


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libspecdraft.so is missing (%s): run `python -m paper_2404_19124_amd.build`; "
                               "there is no fallback path" % LIB_PATH)
        l = C.CDLL(LIB_PATH)
        l.spec_create.restype = C.c_int
        l.spec_create.argtypes = [C.POINTER(spec_config_t), C.POINTER(spec_weights_t), C.c_void_p,
                                  C.POINTER(C.c_void_p)]
        l.spec_destroy.restype = None
        l.spec_destroy.argtypes = [C.c_void_p]
        l.spec_draft.restype = C.c_int
        l.spec_draft.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_int32,
                                 C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(spec_debug_t), C.c_void_p]
        l.spec_verify.restype = C.c_int
        l.spec_verify.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                  C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        l.spec_head_logp.restype = C.c_int
        l.spec_head_logp.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        l.spec_model_scalars.restype = C.c_int
        l.spec_model_scalars.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(C.c_float)]
        l.spec_profile_enable.restype = C.c_int
        l.spec_profile_enable.argtypes = [C.c_void_p, C.c_int32]
        l.spec_profile_read.restype = C.c_int
        l.spec_profile_read.argtypes = [C.c_void_p, C.POINTER(spec_launch_record_t), C.c_int32, C.POINTER(C.c_int32)]
        l.spec_plan_contraction.restype = C.c_int
        l.spec_plan_contraction.argtypes = [C.c_int32] * 6 + [C.POINTER(spec_plan_t)]
        l.spec_set_fused.restype = C.c_int
        l.spec_set_fused.argtypes = [C.c_void_p, C.c_int32]
        l.spec_fused_timeout.restype = C.c_int
        l.spec_fused_timeout.argtypes = [C.c_void_p, C.c_int64]
        l.spec_fused_phase_us.restype = C.c_int
        l.spec_fused_phase_us.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.c_int32, C.POINTER(C.c_int32)]
        l.spec_tree_metadata.restype = C.c_int
        l.spec_tree_metadata.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32] + [C.c_void_p] * 7
        l.spec_advance.restype = C.c_int
        l.spec_advance.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32] + [C.c_void_p] * 6
        l.spec_copy_probe.restype = C.c_int
        l.spec_copy_probe.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        l.spec_last_error.restype = C.c_char_p
        l.spec_last_error.argtypes = []
        l.spec_version.restype = C.c_int
        l.spec_version.argtypes = [C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        _lib = l
    return _lib


def spec_last_error() -> str:
    return lib().spec_last_error().decode()


def _check(status: int) -> None:
    if status != SPEC_OK:
        raise SpecError(status, spec_last_error())


def spec_version():
    a, b = C.c_int32(), C.c_int32()
    _check(lib().spec_version(C.byref(a), C.byref(b)))
    return a.value, b.value


def _dtype_code(name: str) -> int:
    return {"f32": SPEC_F32, "bf16": SPEC_BF16}[name]


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _ptr(t: Optional[torch.Tensor]):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def make_config(n_predict, emb_dim, inner_dim, vocab, weight_dtype, max_batch, max_top_k, state_weight=-1.0,
                emb_weight=-1.0, ln_eps=1e-5) -> spec_config_t:
    cfg = spec_config_t()
    cfg.n_predict, cfg.emb_dim, cfg.inner_dim, cfg.vocab = n_predict, emb_dim, inner_dim, vocab
    cfg.weight_dtype = _dtype_code(weight_dtype) if isinstance(weight_dtype, str) else int(weight_dtype)
    cfg.state_weight, cfg.emb_weight, cfg.ln_eps = state_weight, emb_weight, ln_eps
    cfg.max_batch = max_batch
    for i, k in enumerate(list(max_top_k)[:SPEC_MAX_STAGES]):
        cfg.max_top_k[i] = int(k)
    return cfg


class SpecModel:
    """Owner of a spec_model_t*.  Keeps the borrowed tensors alive."""

    def __init__(self, cfg: spec_config_t, weights: Dict[str, List[torch.Tensor]], stream=None):
        n = cfg.n_predict
        self.cfg = cfg
        self._keep = {k: [t.contiguous() for t in weights[k]] for k in ("emb", "ln_gamma", "ln_beta")}
        tmp = {k: [t.contiguous() for t in weights[k]] for k in ("proj", "head")}
        w = spec_weights_t()
        arrays = {}
        for key in ("proj", "emb", "head", "ln_gamma", "ln_beta"):
            src = tmp[key] if key in tmp else self._keep[key]
            if len(src) != n:
                raise ValueError("weights[%s] needs %d stages" % (key, n))
            arr = (C.c_void_p * n)(*[t.data_ptr() for t in src])
            arrays[key] = arr
            setattr(w, key, C.cast(arr, C.POINTER(C.c_void_p)))
        handle = C.c_void_p()
        _check(lib().spec_create(C.byref(cfg), C.byref(w), _stream_ptr(stream), C.byref(handle)))
        self.handle = handle
        del tmp  # proj / head were copied by the library

    def scalars(self):
        a, b, c = C.c_float(), C.c_float(), C.c_float()
        _check(lib().spec_model_scalars(self.handle, C.byref(a), C.byref(b), C.byref(c)))
        return a.value, b.value, c.value

    def close(self):
        if getattr(self, "handle", None):
            lib().spec_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def spec_draft(model: SpecModel, state: torch.Tensor, last_tok: torch.Tensor, top_k: Sequence[int], B: int,
               cand_tokens: torch.Tensor, cand_scores: torch.Tensor, cand_leaf: torch.Tensor,
               dbg: Optional[Dict[str, torch.Tensor]] = None, stream=None) -> None:
    """Enqueues one draft.  All tensors are caller-allocated device tensors."""
    batch = state.shape[0]
    tk = (C.c_int32 * len(top_k))(*[int(k) for k in top_k])
    d = None
    if dbg is not None:
        d = spec_debug_t(_ptr(dbg.get("stage_state")), _ptr(dbg.get("topk_tok")), _ptr(dbg.get("topk_logp")),
                         _ptr(dbg.get("row_lse")))
    _check(lib().spec_draft(model.handle, _ptr(state), _ptr(last_tok), batch, tk, int(B), _ptr(cand_tokens),
                            _ptr(cand_scores), _ptr(cand_leaf), C.byref(d) if d is not None else None,
                            _stream_ptr(stream)))


def spec_verify(base_logits: torch.Tensor, cand_tokens: torch.Tensor, greedy: torch.Tensor, accept_len: torch.Tensor,
                best_cand: torch.Tensor, out_tokens: torch.Tensor, n_out: torch.Tensor,
                accept_all: Optional[torch.Tensor] = None, stream=None) -> None:
    """Enqueues one verify.  base_logits [batch, B, n+1, V] float32 or bfloat16."""
    b, B, n1, V = base_logits.shape
    code = {torch.float32: SPEC_F32, torch.bfloat16: SPEC_BF16}.get(base_logits.dtype, -1)
    _check(lib().spec_verify(_ptr(base_logits), code, _ptr(cand_tokens), b, B, n1 - 1, V, _ptr(greedy),
                             _ptr(accept_len), _ptr(best_cand), _ptr(out_tokens), _ptr(n_out), _ptr(accept_all),
                             _stream_ptr(stream)))


def spec_profile_enable(model: SpecModel, capacity: int) -> None:
    _check(lib().spec_profile_enable(model.handle, int(capacity)))


def spec_profile_read(model: SpecModel, cap: int = 65536):
    """Returns a list of dicts (kernel, rows, weight_rows, k, ms), in launch order."""
    buf = (spec_launch_record_t * cap)()
    n = C.c_int32()
    _check(lib().spec_profile_read(model.handle, buf, cap, C.byref(n)))
    return [dict(kernel=r.kernel, rows=r.rows, weight_rows=r.weight_rows, k=r.k, ms=r.ms) for r in buf[:n.value]]


def spec_set_fused(model: SpecModel, enable: bool) -> None:
    _check(lib().spec_set_fused(model.handle, 1 if enable else 0))


def spec_fused_timeout(model: SpecModel, microseconds: int) -> None:
    _check(lib().spec_fused_timeout(model.handle, int(microseconds)))


def spec_fused_phase_us(model: SpecModel):
    """Phase durations (us) of the last fused draft launch; [] if none has run."""
    buf = (C.c_float * 32)()
    n = C.c_int32()
    _check(lib().spec_fused_phase_us(model.handle, buf, 32, C.byref(n)))
    return [float(x) for x in buf[:n.value]]


def spec_tree_metadata(cand_tokens: torch.Tensor, node_tok: torch.Tensor, node_parent: torch.Tensor,
                       node_depth: torch.Tensor, n_nodes: torch.Tensor, cand_node: torch.Tensor,
                       mask: Optional[torch.Tensor] = None, stream=None) -> None:
    b, Bc, n = cand_tokens.shape
    _check(lib().spec_tree_metadata(_ptr(cand_tokens), b, Bc, n, _ptr(node_tok), _ptr(node_parent), _ptr(node_depth),
                                    _ptr(n_nodes), _ptr(cand_node), _ptr(mask) if mask is not None else None,
                                    _stream_ptr(stream)))


def spec_advance(hidden: torch.Tensor, best_cand: torch.Tensor, accept_len: torch.Tensor, out_tokens: torch.Tensor,
                 next_state: torch.Tensor, next_tok: torch.Tensor, stream=None) -> None:
    b, Bc, n1, E = hidden.shape
    dtype = {torch.float32: SPEC_F32, torch.bfloat16: SPEC_BF16}[hidden.dtype]
    _check(lib().spec_advance(_ptr(hidden), dtype, b, Bc, n1 - 1, E, _ptr(best_cand), _ptr(accept_len),
                              _ptr(out_tokens), _ptr(next_state), _ptr(next_tok), _stream_ptr(stream)))


def spec_plan_contraction(rows: int, k: int, n_head: int, k_top: int, n_proj: int, n_cu: int = 256) -> dict:
    """The launch plan of one contraction (host-only: needs no GPU)."""
    out = spec_plan_t()
    _check(lib().spec_plan_contraction(int(rows), int(k), int(n_head), int(k_top), int(n_proj), int(n_cu), C.byref(out)))
    return {name: int(getattr(out, name)) for name, _ in spec_plan_t._fields_}


def spec_copy_probe(src: torch.Tensor, dst: torch.Tensor, stream=None) -> int:
    """One plain copy launch src -> dst (same byte size); returns the bytes copied."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("src and dst differ in size")
    _check(lib().spec_copy_probe(_ptr(src), _ptr(dst), nbytes, _stream_ptr(stream)))
    return nbytes


def spec_head_logp(model: SpecModel, stage: int, states: torch.Tensor, logp: torch.Tensor, stream=None) -> None:
    _check(lib().spec_head_logp(model.handle, int(stage), _ptr(states), states.shape[0], _ptr(logp),
                                _stream_ptr(stream)))
