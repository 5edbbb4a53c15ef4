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

EXPORTS = ["spec_create", "spec_destroy", "spec_draft", "spec_draft_static", "spec_draft_dynamic", "spec_verify", "spec_verify_dynamic", "spec_head_logp", "spec_model_scalars",
           "spec_profile_enable", "spec_profile_read", "spec_copy_probe", "spec_tree_metadata", "spec_advance", "spec_plan_contraction", "spec_last_error", "spec_version"]


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
                                               "parts", "k_split", "workgroups", "lds_bytes", "proj_apart")]


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
        l.spec_draft_static.restype = C.c_int
        l.spec_draft_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_int32,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        l.spec_draft_dynamic.restype = C.c_int
        l.spec_draft_dynamic.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(C.c_int32),
                                         C.POINTER(C.c_int32), C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.POINTER(spec_debug_t), C.c_void_p]
        l.spec_verify_dynamic.restype = C.c_int
        l.spec_verify_dynamic.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                          C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_void_p]
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


_TORCH_DTYPE = {SPEC_F32: torch.float32, SPEC_BF16: torch.bfloat16}
_CHECK_DEVICE = True   # the CPU-only tests of _require switch the device check off to reach the others


def _require(t, name: str, dtype: torch.dtype, shape: Optional[Sequence[int]] = None, optional: bool = False) -> None:
    """Host-side check of a tensor argument before its address crosses the boundary: the library reads
    raw pointers, so a wrong element type, a view with strides or a short buffer would be read (or
    written) out of bounds on the device.  Raises ValueError."""
    if t is None:
        if optional:
            return
        raise ValueError("%s is required" % name)
    if not isinstance(t, torch.Tensor):
        raise ValueError("%s must be a torch.Tensor" % name)
    if t.dtype != dtype:
        raise ValueError("%s must have dtype %s, got %s" % (name, dtype, t.dtype))
    if shape is not None and tuple(t.shape) != tuple(int(x) for x in shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if _CHECK_DEVICE and not t.is_cuda:
        raise ValueError("%s must be a device tensor" % name)


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
        wdt = _TORCH_DTYPE.get(cfg.weight_dtype)
        if wdt is None:
            raise ValueError("weight_dtype %d is neither SPEC_F32 nor SPEC_BF16" % cfg.weight_dtype)
        for key in ("proj", "emb", "head", "ln_gamma", "ln_beta"):
            if key not in weights or len(weights[key]) != n:
                raise ValueError("weights[%s] needs %d stages" % (key, n))
        for i in range(n):
            in_i = cfg.emb_dim if i == 0 else cfg.inner_dim
            for key, dt, shape in (("proj", wdt, (cfg.inner_dim, in_i)), ("emb", wdt, (cfg.vocab, cfg.inner_dim)),
                                   ("head", wdt, (cfg.vocab, cfg.inner_dim)),
                                   ("ln_gamma", torch.float32, (cfg.inner_dim,)),
                                   ("ln_beta", torch.float32, (cfg.inner_dim,))):
                t = weights[key][i]
                if not isinstance(t, torch.Tensor) or t.dtype != dt or tuple(t.shape) != shape or not t.is_cuda:
                    raise ValueError("weights[%s][%d] must be a device tensor of dtype %s and shape %s"
                                     % (key, i, dt, shape))
        self._keep = {k: [t.contiguous() for t in weights[k]] for k in ("emb", "ln_gamma", "ln_beta")}
        tmp = {k: [t.contiguous() for t in weights[k]] for k in ("proj", "head")}
        w = spec_weights_t()
        arrays = {}
        for key in ("proj", "emb", "head", "ln_gamma", "ln_beta"):
            src = tmp[key] if key in tmp else self._keep[key]
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
    cfg = model.cfg
    n, D = cfg.n_predict, cfg.inner_dim
    wdt = _TORCH_DTYPE[cfg.weight_dtype]
    top_k = [int(k) for k in top_k]
    if len(top_k) != n:
        raise ValueError("top_k needs %d entries, got %d" % (n, len(top_k)))
    if not isinstance(state, torch.Tensor) or state.dim() != 2:
        raise ValueError("state must be a [batch, emb_dim] tensor")
    batch, B = int(state.shape[0]), int(B)
    _require(state, "state", wdt, (batch, cfg.emb_dim))
    _require(last_tok, "last_tok", torch.int32, (batch,))
    _require(cand_tokens, "cand_tokens", torch.int32, (batch, B, n))
    _require(cand_scores, "cand_scores", torch.float32, (batch, B))
    _require(cand_leaf, "cand_leaf", torch.int32, (batch, B))
    if dbg is not None:
        rows, r = [], batch
        for k in top_k:
            rows.append(r)
            r *= max(k, 0)
        sum_rows, sum_rk = sum(rows), sum(r_ * k for r_, k in zip(rows, top_k))
        _require(dbg.get("stage_state"), "dbg[stage_state]", wdt, (sum_rows, D), optional=True)
        _require(dbg.get("topk_tok"), "dbg[topk_tok]", torch.int32, (sum_rk,), optional=True)
        _require(dbg.get("topk_logp"), "dbg[topk_logp]", torch.float32, (sum_rk,), optional=True)
        _require(dbg.get("row_lse"), "dbg[row_lse]", torch.float32, (sum_rows,), optional=True)
    tk = (C.c_int32 * n)(*top_k)
    d = None
    if dbg is not None:
        d = spec_debug_t(_ptr(dbg.get("stage_state")), _ptr(dbg.get("topk_tok")), _ptr(dbg.get("topk_logp")),
                         _ptr(dbg.get("row_lse")))
    _check(lib().spec_draft(model.handle, _ptr(state), _ptr(last_tok), batch, tk, int(B), _ptr(cand_tokens),
                            _ptr(cand_scores), _ptr(cand_leaf), C.byref(d) if d is not None else None,
                            _stream_ptr(stream)))


def spec_draft_static(model: SpecModel, state: torch.Tensor, last_tok: torch.Tensor, top_k: Sequence[int], B: int,
                      cand_tokens: torch.Tensor, cand_scores: torch.Tensor, cand_leaf: torch.Tensor,
                      stream=None) -> None:
    """spec_draft with the call's workspace in the library's static device array (no allocation)."""
    cfg = model.cfg
    n = cfg.n_predict
    wdt = _TORCH_DTYPE[cfg.weight_dtype]
    top_k = [int(k) for k in top_k]
    if len(top_k) != n:
        raise ValueError("top_k needs %d entries, got %d" % (n, len(top_k)))
    if not isinstance(state, torch.Tensor) or state.dim() != 2:
        raise ValueError("state must be a [batch, emb_dim] tensor")
    batch, B = int(state.shape[0]), int(B)
    _require(state, "state", wdt, (batch, cfg.emb_dim))
    _require(last_tok, "last_tok", torch.int32, (batch,))
    _require(cand_tokens, "cand_tokens", torch.int32, (batch, B, n))
    _require(cand_scores, "cand_scores", torch.float32, (batch, B))
    _require(cand_leaf, "cand_leaf", torch.int32, (batch, B))
    tk = (C.c_int32 * n)(*top_k)
    _check(lib().spec_draft_static(model.handle, _ptr(state), _ptr(last_tok), batch, tk, B, _ptr(cand_tokens),
                                   _ptr(cand_scores), _ptr(cand_leaf), _stream_ptr(stream)))


def dynamic_rows(top_k_seq: Sequence[Sequence[int]], B_seq: Sequence[int]):
    """Row bookkeeping of a spec_draft_dynamic call (argument marshalling only): rows per stage over the
    active sequences, the widest branching per stage, and per sequence its first row at every stage."""
    n = len(top_k_seq[0])
    rows, kw, first = [0] * n, [1] * n, []
    for ks, Bq in zip(top_k_seq, B_seq):
        first.append(list(rows))
        if Bq == 0:
            continue
        cnt = 1
        for i, k in enumerate(ks):
            rows[i] += cnt
            kw[i] = max(kw[i], int(k))
            cnt *= int(k)
    return rows, kw, first


def spec_draft_dynamic(model: SpecModel, state: torch.Tensor, last_tok: torch.Tensor,
                       top_k_seq: Sequence[Sequence[int]], B_seq: Sequence[int], cand_tokens: torch.Tensor,
                       cand_scores: torch.Tensor, cand_leaf: torch.Tensor, n_cand: torch.Tensor,
                       dbg: Optional[Dict[str, torch.Tensor]] = None, stream=None) -> None:
    """Enqueues one draft with an own tree (top_k_seq[q]) and candidate count (B_seq[q], 0 = off) per sequence."""
    cfg = model.cfg
    n, D = cfg.n_predict, cfg.inner_dim
    wdt = _TORCH_DTYPE[cfg.weight_dtype]
    if not isinstance(state, torch.Tensor) or state.dim() != 2:
        raise ValueError("state must be a [batch, emb_dim] tensor")
    batch = int(state.shape[0])
    top_k_seq = [[int(k) for k in ks] for ks in top_k_seq]
    B_seq = [int(x) for x in B_seq]
    if len(top_k_seq) != batch or len(B_seq) != batch or any(len(ks) != n for ks in top_k_seq):
        raise ValueError("top_k_seq must be [batch][%d] and B_seq [batch]" % n)
    if not isinstance(cand_tokens, torch.Tensor) or cand_tokens.dim() != 3:
        raise ValueError("cand_tokens must be a [batch, B_pad, n_predict] tensor")
    B_pad = int(cand_tokens.shape[1])
    _require(state, "state", wdt, (batch, cfg.emb_dim))
    _require(last_tok, "last_tok", torch.int32, (batch,))
    _require(cand_tokens, "cand_tokens", torch.int32, (batch, B_pad, n))
    _require(cand_scores, "cand_scores", torch.float32, (batch, B_pad))
    _require(cand_leaf, "cand_leaf", torch.int32, (batch, B_pad))
    _require(n_cand, "n_cand", torch.int32, (batch,))
    d = None
    if dbg is not None:
        rows, kw, _ = dynamic_rows(top_k_seq, B_seq)
        sum_rows, sum_rk = sum(rows), sum(r * k for r, k in zip(rows, kw))
        _require(dbg.get("stage_state"), "dbg[stage_state]", wdt, (sum_rows, D), optional=True)
        _require(dbg.get("topk_tok"), "dbg[topk_tok]", torch.int32, (sum_rk,), optional=True)
        _require(dbg.get("topk_logp"), "dbg[topk_logp]", torch.float32, (sum_rk,), optional=True)
        _require(dbg.get("row_lse"), "dbg[row_lse]", torch.float32, (sum_rows,), optional=True)
        d = spec_debug_t(_ptr(dbg.get("stage_state")), _ptr(dbg.get("topk_tok")), _ptr(dbg.get("topk_logp")),
                         _ptr(dbg.get("row_lse")))
    tk = (C.c_int32 * (batch * n))(*[k for ks in top_k_seq for k in ks])
    bs = (C.c_int32 * batch)(*B_seq)
    _check(lib().spec_draft_dynamic(model.handle, _ptr(state), _ptr(last_tok), batch, tk, bs, B_pad, _ptr(cand_tokens),
                                    _ptr(cand_scores), _ptr(cand_leaf), _ptr(n_cand),
                                    C.byref(d) if d is not None else None, _stream_ptr(stream)))


def spec_verify_dynamic(base_logits: torch.Tensor, cand_tokens: torch.Tensor, n_cand: torch.Tensor,
                        greedy: torch.Tensor, accept_len: torch.Tensor, best_cand: torch.Tensor,
                        out_tokens: torch.Tensor, n_out: torch.Tensor, accept_all: Optional[torch.Tensor] = None,
                        stream=None) -> None:
    """Enqueues one verify in which sequence q has n_cand[q] candidates (0 = speculation off)."""
    if not isinstance(base_logits, torch.Tensor) or base_logits.dim() != 4:
        raise ValueError("base_logits must be a [batch, B, n_predict + 1, vocab] tensor")
    b, B, n1, V = (int(x) for x in base_logits.shape)
    code = {torch.float32: SPEC_F32, torch.bfloat16: SPEC_BF16}.get(base_logits.dtype, -1)
    if code < 0:
        raise ValueError("base_logits must be float32 or bfloat16, got %s" % base_logits.dtype)
    _require(base_logits, "base_logits", base_logits.dtype)
    _require(cand_tokens, "cand_tokens", torch.int32, (b, B, n1 - 1))
    _require(n_cand, "n_cand", torch.int32, (b,))
    _require(greedy, "greedy", torch.int32, (b, B, n1))
    _require(accept_len, "accept_len", torch.int32, (b,))
    _require(best_cand, "best_cand", torch.int32, (b,))
    _require(out_tokens, "out_tokens", torch.int32, (b, n1))
    _require(n_out, "n_out", torch.int32, (b,))
    _require(accept_all, "accept_all", torch.int32, (b, B), optional=True)
    _check(lib().spec_verify_dynamic(_ptr(base_logits), code, _ptr(cand_tokens), _ptr(n_cand), b, B, n1 - 1, V,
                                     _ptr(greedy), _ptr(accept_len), _ptr(best_cand), _ptr(out_tokens), _ptr(n_out),
                                     _ptr(accept_all), _stream_ptr(stream)))


def spec_verify(base_logits: torch.Tensor, cand_tokens: torch.Tensor, greedy: torch.Tensor, accept_len: torch.Tensor,
                best_cand: torch.Tensor, out_tokens: torch.Tensor, n_out: torch.Tensor,
                accept_all: Optional[torch.Tensor] = None, stream=None) -> None:
    """Enqueues one verify.  base_logits [batch, B, n+1, V] float32 or bfloat16."""
    if not isinstance(base_logits, torch.Tensor) or base_logits.dim() != 4:
        raise ValueError("base_logits must be a [batch, B, n_predict + 1, vocab] tensor")
    b, B, n1, V = (int(x) for x in base_logits.shape)
    code = {torch.float32: SPEC_F32, torch.bfloat16: SPEC_BF16}.get(base_logits.dtype, -1)
    if code < 0:
        raise ValueError("base_logits must be float32 or bfloat16, got %s" % base_logits.dtype)
    _require(base_logits, "base_logits", base_logits.dtype)
    _require(cand_tokens, "cand_tokens", torch.int32, (b, B, n1 - 1))
    _require(greedy, "greedy", torch.int32, (b, B, n1))
    _require(accept_len, "accept_len", torch.int32, (b,))
    _require(best_cand, "best_cand", torch.int32, (b,))
    _require(out_tokens, "out_tokens", torch.int32, (b, n1))
    _require(n_out, "n_out", torch.int32, (b,))
    _require(accept_all, "accept_all", torch.int32, (b, B), optional=True)
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


def spec_tree_metadata(cand_tokens: torch.Tensor, node_tok: torch.Tensor, node_parent: torch.Tensor,
                       node_depth: torch.Tensor, n_nodes: torch.Tensor, cand_node: torch.Tensor,
                       mask: Optional[torch.Tensor] = None, stream=None) -> None:
    if not isinstance(cand_tokens, torch.Tensor) or cand_tokens.dim() != 3:
        raise ValueError("cand_tokens must be a [batch, B, n_predict] tensor")
    b, Bc, n = (int(x) for x in cand_tokens.shape)
    M = Bc * n
    _require(cand_tokens, "cand_tokens", torch.int32)
    _require(node_tok, "node_tok", torch.int32, (b, M))
    _require(node_parent, "node_parent", torch.int32, (b, M))
    _require(node_depth, "node_depth", torch.int32, (b, M))
    _require(n_nodes, "n_nodes", torch.int32, (b,))
    _require(cand_node, "cand_node", torch.int32, (b, Bc, n))
    _require(mask, "mask", torch.uint8, (b, M, M), optional=True)
    _check(lib().spec_tree_metadata(_ptr(cand_tokens), b, Bc, n, _ptr(node_tok), _ptr(node_parent), _ptr(node_depth),
                                    _ptr(n_nodes), _ptr(cand_node), _ptr(mask) if mask is not None else None,
                                    _stream_ptr(stream)))


def spec_advance(hidden: torch.Tensor, best_cand: torch.Tensor, accept_len: torch.Tensor, out_tokens: torch.Tensor,
                 next_state: torch.Tensor, next_tok: torch.Tensor, stream=None) -> None:
    if not isinstance(hidden, torch.Tensor) or hidden.dim() != 4:
        raise ValueError("hidden must be a [batch, B, n_predict + 1, emb_dim] tensor")
    b, Bc, n1, E = (int(x) for x in hidden.shape)
    dtype = {torch.float32: SPEC_F32, torch.bfloat16: SPEC_BF16}.get(hidden.dtype, -1)
    if dtype < 0:
        raise ValueError("hidden must be float32 or bfloat16, got %s" % hidden.dtype)
    _require(hidden, "hidden", hidden.dtype)
    _require(best_cand, "best_cand", torch.int32, (b,))
    _require(accept_len, "accept_len", torch.int32, (b,))
    _require(out_tokens, "out_tokens", torch.int32, (b, n1))
    _require(next_state, "next_state", hidden.dtype, (b, E))
    _require(next_tok, "next_tok", torch.int32, (b,))
    _check(lib().spec_advance(_ptr(hidden), dtype, b, Bc, n1 - 1, E, _ptr(best_cand), _ptr(accept_len),
                              _ptr(out_tokens), _ptr(next_state), _ptr(next_tok), _stream_ptr(stream)))


def spec_plan_contraction(rows: int, k: int, n_head: int, k_top: int, n_proj: int, n_cu: int = 256) -> dict:
    """The launch plan of one contraction (host-only: needs no GPU)."""
    out = spec_plan_t()
    _check(lib().spec_plan_contraction(int(rows), int(k), int(n_head), int(k_top), int(n_proj), int(n_cu), C.byref(out)))
    return {name: int(getattr(out, name)) for name, _ in spec_plan_t._fields_}


def spec_copy_probe(src: torch.Tensor, dst: torch.Tensor, stream=None) -> int:
    """One plain copy launch src -> dst (same byte size); returns the bytes copied."""
    _require(src, "src", src.dtype)
    _require(dst, "dst", dst.dtype)
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("src and dst differ in size")
    _check(lib().spec_copy_probe(_ptr(src), _ptr(dst), nbytes, _stream_ptr(stream)))
    return nbytes


def spec_head_logp(model: SpecModel, stage: int, states: torch.Tensor, logp: torch.Tensor, stream=None) -> None:
    cfg = model.cfg
    if not isinstance(states, torch.Tensor) or states.dim() != 2:
        raise ValueError("states must be a [rows, inner_dim] tensor")
    _require(states, "states", _TORCH_DTYPE[cfg.weight_dtype], (states.shape[0], cfg.inner_dim))
    _require(logp, "logp", torch.float32, (states.shape[0], cfg.vocab))
    _check(lib().spec_head_logp(model.handle, int(stage), _ptr(states), states.shape[0], _ptr(logp),
                                _stream_ptr(stream)))
