"""Convenience layer over the binding for tests, the smoke check and the
benchmark: builds a model for a workload, owns the output tensors of a step and
enqueues draft / verify.  No arithmetic of the method happens here."""
from __future__ import annotations

from typing import Dict, List, Optional

import torch

from . import binding as B
from .workloads import Workload


class Step:
    """One draft + verify step of a workload on the current CUDA (HIP) device."""

    def __init__(self, wl: Workload, weights: Dict[str, List[torch.Tensor]], debug: bool = False,
                 state_weight: float = -1.0, emb_weight: float = -1.0, ln_eps: float = 1e-5,
                 max_batch: Optional[int] = None, max_top_k=None):
        self.wl = wl
        dev = weights["emb"][0].device
        cfg = B.make_config(wl.n_predict, wl.emb_dim, wl.inner_dim, wl.vocab, wl.weight_dtype,
                            max_batch or wl.batch, max_top_k or wl.top_k, state_weight, emb_weight, ln_eps)
        self.model = B.SpecModel(cfg, weights)
        b, n, Bc = wl.batch, wl.n_predict, wl.B
        i32 = dict(dtype=torch.int32, device=dev)
        self.cand_tokens = torch.empty((b, Bc, n), **i32)
        self.cand_scores = torch.empty((b, Bc), dtype=torch.float32, device=dev)
        self.cand_leaf = torch.empty((b, Bc), **i32)
        self.greedy = torch.empty((b, Bc, n + 1), **i32)
        self.accept_len = torch.empty((b,), **i32)
        self.best_cand = torch.empty((b,), **i32)
        self.out_tokens = torch.empty((b, n + 1), **i32)
        self.n_out = torch.empty((b,), **i32)
        self.accept_all = torch.empty((b, Bc), **i32)
        self.dbg = None
        if debug:
            rows = wl.rows()
            sum_rows = sum(rows)
            sum_rk = sum(r * k for r, k in zip(rows, wl.top_k))
            sdt = torch.bfloat16 if wl.weight_dtype == "bf16" else torch.float32
            self.dbg = {
                "stage_state": torch.zeros((sum_rows, wl.inner_dim), dtype=sdt, device=dev),
                "topk_tok": torch.zeros((sum_rk,), **i32),
                "topk_logp": torch.zeros((sum_rk,), dtype=torch.float32, device=dev),
                "row_lse": torch.zeros((sum_rows,), dtype=torch.float32, device=dev),
            }

    def draft(self, state: torch.Tensor, last_tok: torch.Tensor, stream=None) -> None:
        B.spec_draft(self.model, state, last_tok, self.wl.top_k, self.wl.B, self.cand_tokens, self.cand_scores,
                     self.cand_leaf, self.dbg, stream)

    def verify(self, base_logits: torch.Tensor, cand_tokens: Optional[torch.Tensor] = None, stream=None) -> None:
        B.spec_verify(base_logits, self.cand_tokens if cand_tokens is None else cand_tokens, self.greedy,
                      self.accept_len, self.best_cand, self.out_tokens, self.n_out, self.accept_all, stream)

    def debug_tables(self):
        """Per-stage views of the debug tensors: states, tok, logp, lse."""
        wl = self.wl
        out = {"states": [], "tok": [], "logp": [], "lse": []}
        ro, ko = 0, 0
        for r, k in zip(wl.rows(), wl.top_k):
            out["states"].append(self.dbg["stage_state"][ro:ro + r])
            out["lse"].append(self.dbg["row_lse"][ro:ro + r])
            out["tok"].append(self.dbg["topk_tok"][ko:ko + r * k].view(r, k))
            out["logp"].append(self.dbg["topk_logp"][ko:ko + r * k].view(r, k))
            ro += r
            ko += r * k
        return out

    def close(self):
        self.model.close()
