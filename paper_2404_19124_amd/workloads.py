"""Seeded synthetic inputs for the draft + verify step.

This module holds none of the method's arithmetic: it only draws random tensors
with the shapes and value distributions of the paper's workloads (Sec. 4: latent
width 4096, base widths 4096 / 5120, 32k vocabulary, 3..7 stages, trees such as
6/3/2 pruned to k candidates).  Both the CPU oracle's tests and the HIP path's
tests / benchmark draw their inputs here, so that they see identical tensors.

Nothing of the paper's datasets, prompts or trained weights is used or needed:
the cost of the path depends on shapes only.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Tuple

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    emb_dim: int          # E: width of the base model's hidden vector
    inner_dim: int        # D: latent width of the speculator
    vocab: int            # V
    n_predict: int        # n: stages / speculated tokens
    top_k: Tuple[int, ...]
    B: int                # candidates kept per sequence
    batch: int
    weight_dtype: str     # "f32" | "bf16": projection / head / embedding / state storage
    logits_dtype: str     # "f32" | "bf16": base-model logits
    p_boost: float
    seed: int = 0
    emb_std: float = 0.02   # tests raise it so that the sampled token visibly steers the state

    @property
    def leaves(self) -> int:
        out = 1
        for k in self.top_k:
            out *= k
        return out

    def rows(self) -> List[int]:
        """Head rows R_i per stage: batch * prod_{j<i} k_j."""
        out, r = [], self.batch
        for k in self.top_k:
            out.append(r)
            r *= k
        return out

    def param_count(self) -> int:
        n, E, D, V = self.n_predict, self.emb_dim, self.inner_dim, self.vocab
        return D * E + (n - 1) * D * D + 2 * n * V * D + 2 * n * D

    def algorithmic_bytes(self) -> Dict[str, int]:
        """Bytes one step must move: every projection and head weight once, one
        embedding row and one state row per node, the base logits once."""
        w = 2 if self.weight_dtype == "bf16" else 4
        l = 2 if self.logits_dtype == "bf16" else 4
        n, E, D, V = self.n_predict, self.emb_dim, self.inner_dim, self.vocab
        proj = (D * E + (n - 1) * D * D) * w
        head = n * V * D * w
        rows = sum(self.rows())
        emb = rows * D * w
        logits = self.batch * self.B * (n + 1) * V * l
        return {"proj": proj, "head": head, "emb_rows": emb, "base_logits": logits,
                "total": proj + head + emb + logits}

    def contraction_flops(self) -> int:
        n, E, D, V = self.n_predict, self.emb_dim, self.inner_dim, self.vocab
        R = self.rows()
        P = [self.batch] + R[:-1]
        head = sum(2 * r * V * D for r in R)
        proj = 2 * P[0] * D * E + sum(2 * p * D * D for p in P[1:])
        return head + proj


# The five configurations of the build's baseline description, in order, then the code-model shapes.
WORKLOADS: Dict[str, Workload] = {
    "tiny_b1": Workload("tiny_b1", 256, 256, 1024, 3, (4, 3, 2), 24, 1, "f32", "f32", 0.6),
    "llama7b_b1": Workload("llama7b_b1", 4096, 4096, 32000, 3, (5, 3, 2), 16, 1, "bf16", "f32", 0.6),
    "llama7b_b64": Workload("llama7b_b64", 4096, 4096, 32000, 3, (5, 3, 2), 16, 64, "bf16", "f32", 0.6),
    "llama13b_b16": Workload("llama13b_b16", 5120, 4096, 32000, 3, (6, 4, 3), 32, 16, "bf16", "f32", 0.5),
    "large70b_b32": Workload("large70b_b32", 8192, 3072, 128256, 4, (6, 4, 3, 2), 64, 32, "bf16", "bf16", 0.5),
    # Code-model shapes (Sec. 4.3, 4.4 of the paper): 7 heads on a 5120-wide base with a 32016-token
    # vocabulary, 5 heads on a 6144-wide base with 49152 tokens; k = 1 chains (the setting the paper
    # finds best on a loaded server) and a small tree.  Code is predictable: high acceptance rate.
    "code13b_k1_b1": Workload("code13b_k1_b1", 5120, 4096, 32016, 7, (1,) * 7, 1, 1, "bf16", "f32", 0.8),
    "code13b_tree_b4": Workload("code13b_tree_b4", 5120, 4096, 32016, 7, (2, 2, 1, 1, 1, 1, 1), 4, 4, "bf16", "f32",
                                0.8),
    "code20b_k1_b8": Workload("code20b_k1_b8", 6144, 4096, 49152, 5, (1,) * 5, 1, 8, "bf16", "f32", 0.8),
}


def small_variant(wl: Workload, **kw) -> Workload:
    return replace(wl, **kw)


def _tdtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def make_generator(seed: int, device: str = "cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def make_speculator(wl: Workload, gen: torch.Generator, device: str = "cpu",
                    ln_affine: str = "identity") -> Dict[str, list]:
    """Weights N(0, 0.02) drawn in float32 then rounded to the storage type, in
    the order proj_i, emb_i, head_i for i = 1..n.  LayerNorm gamma = 1, beta = 0
    unless ln_affine == "random" (gamma = 1 + 0.1 N, beta = 0.1 N), which tests
    use so that a dropped gamma / beta cannot go unnoticed."""
    dt = _tdtype(wl.weight_dtype)
    w = {"proj": [], "emb": [], "head": [], "ln_gamma": [], "ln_beta": []}
    for i in range(wl.n_predict):
        in_dim = wl.emb_dim if i == 0 else wl.inner_dim
        for key, shape in (("proj", (wl.inner_dim, in_dim)), ("emb", (wl.vocab, wl.inner_dim)),
                           ("head", (wl.vocab, wl.inner_dim))):
            std = wl.emb_std if key == "emb" else 0.02
            t = torch.empty(shape, dtype=torch.float32, device=device).normal_(0.0, std, generator=gen)
            w[key].append(t.to(dt))
            del t
    for i in range(wl.n_predict):
        if ln_affine == "random":
            g = 1.0 + 0.1 * torch.randn(wl.inner_dim, generator=gen, device=device)
            b = 0.1 * torch.randn(wl.inner_dim, generator=gen, device=device)
        else:
            g = torch.ones(wl.inner_dim, device=device)
            b = torch.zeros(wl.inner_dim, device=device)
        w["ln_gamma"].append(g.float())
        w["ln_beta"].append(b.float())
    return w


def make_draft_inputs(wl: Workload, gen: torch.Generator, device: str = "cpu"):
    """Base-model state N(0,1) [batch, E] in the storage type, last token
    uniform in [0, V)."""
    state = torch.randn(wl.batch, wl.emb_dim, generator=gen, device=device).to(_tdtype(wl.weight_dtype))
    last_tok = torch.randint(0, wl.vocab, (wl.batch,), generator=gen, device=device, dtype=torch.int32)
    return state, last_tok


def make_base_logits(wl: Workload, cand_tokens: torch.Tensor, gen: torch.Generator,
                     device: str = "cpu", batch_chunk: int = 4) -> torch.Tensor:
    """Stand-in for the base model's output over the flattened candidates:
    N(0,1) noise [batch, B, n+1, V]; at positions 0..n-1 the speculated token's
    logit gets +3 with probability p_boost, so that acceptances occur.  Position
    n has no speculated token and is never boosted.  The boost is added in
    float32, then the tensor is rounded to the logits type."""
    b, B, n, V = wl.batch, wl.B, wl.n_predict, wl.vocab
    cand = cand_tokens.to(device=device, dtype=torch.int64).reshape(b, B, n)
    out = torch.empty((b, B, n + 1, V), dtype=_tdtype(wl.logits_dtype), device=device)
    mask = torch.rand((b, B, n), generator=gen, device=device) < wl.p_boost
    for q0 in range(0, b, batch_chunk):
        q1 = min(b, q0 + batch_chunk)
        noise = torch.randn((q1 - q0, B, n + 1, V), generator=gen, device=device)
        boost = torch.zeros((q1 - q0, B, n, 1), device=device)
        boost[mask[q0:q1].unsqueeze(-1)] = 3.0
        spec = noise[:, :, :n, :]
        spec.scatter_add_(3, cand[q0:q1].unsqueeze(-1), boost)
        out[q0:q1] = noise.to(out.dtype)
        del noise
    return out


def to_numpy_f32(t: torch.Tensor):
    """Exact upcast of a (possibly bf16, possibly device) tensor for the oracle."""
    return t.detach().to("cpu").float().numpy()


def weights_to_numpy(w: Dict[str, list]) -> Dict[str, list]:
    return {k: [to_numpy_f32(t) for t in v] for k, v in w.items()}
