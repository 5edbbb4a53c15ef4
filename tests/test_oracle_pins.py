"""Pins of the oracle's scalar rules and single-stage functions against closed
forms, invariants and library routines (torch CPU, float64).  None of these
tests touches the HIP path."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import spec_oracle as O


# ---- mix weights (Sec. 4: base state carries 50% of the final state's variance)
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 7])
def test_mix_weights_closed_form(n):
    w_s, w_e = O.mix_weights(n)
    assert abs(w_s ** 2 + w_e ** 2 - 1.0) < 1e-14       # state keeps unit variance
    assert abs(w_s ** (2 * n) - 0.5) < 1e-14            # base share after n stages


def test_mix_weights_printed_values():
    # values derived by hand for n = 3 and n = 4
    assert np.allclose(O.mix_weights(3), (0.8908987, 0.4542021), atol=1e-6)
    assert np.allclose(O.mix_weights(4), (0.9170040, 0.3988785), atol=1e-6)


def test_mix_weights_by_simulation():
    # linear recursion on independent unit-variance vectors: the share of the
    # base vector in the final one is the squared correlation with it.
    rng = np.random.default_rng(0)
    n, dim = 3, 400000
    w_s, w_e = O.mix_weights(n)
    z = rng.standard_normal(dim)
    s = z.copy()
    for _ in range(n):
        s = w_s * s + w_e * rng.standard_normal(dim)
    share = np.corrcoef(z, s)[0, 1] ** 2
    assert abs(s.var() - 1.0) < 0.01
    assert abs(share - 0.5) < 0.01


# ---- bf16 rounding
def test_round_bf16_matches_torch():
    g = torch.Generator().manual_seed(1)
    x = torch.randn(20000, generator=g) * torch.logspace(-6, 6, 20000)
    want = x.to(torch.bfloat16).float().numpy().astype(np.float64)
    got = O.round_bf16(x.numpy().astype(np.float64))
    assert np.array_equal(got, want)


def test_round_bf16_ties_to_even():
    # bf16 has 8 significant bits: spacing 2^-7 in [1, 2)
    assert O.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0                  # tie -> even (down)
    assert O.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2 * 2.0 ** -7   # tie -> even (up)
    assert O.round_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20]))[0] == 1.0 + 2.0 ** -7
    assert O.round_bf16(np.array([-0.3]))[0] == -0.30078125
    assert O.round_bf16(np.array([0.0]))[0] == 0.0


# ---- LayerNorm
def test_layer_norm_zero_mean_unit_variance():
    rng = np.random.default_rng(2)
    z = rng.standard_normal((7, 256)) * 3.0 + 1.5
    eps = 1e-5
    y = O.layer_norm(z, np.ones(256), np.zeros(256), eps)
    assert np.abs(y.mean(-1)).max() < 1e-12
    # variance is var/(var+eps): one within eps
    want_var = z.var(-1) / (z.var(-1) + eps)
    assert np.allclose(y.var(-1), want_var, rtol=0, atol=1e-12)
    assert np.abs(y.var(-1) - 1.0).max() < 1e-5


def test_layer_norm_matches_torch_with_affine():
    rng = np.random.default_rng(3)
    z = rng.standard_normal((5, 96))
    gam = rng.standard_normal(96)
    bet = rng.standard_normal(96)
    want = F.layer_norm(torch.from_numpy(z), (96,), torch.from_numpy(gam), torch.from_numpy(bet), 1e-5).numpy()
    got = O.layer_norm(z, gam, bet, 1e-5)
    assert np.allclose(got, want, rtol=0, atol=1e-12)


def test_layer_norm_eps_inside_root():
    # a constant row has zero variance: output is exactly beta, finite
    z = np.full((1, 8), 4.0)
    y = O.layer_norm(z, np.full(8, 2.0), np.full(8, 0.25), 1e-5)
    assert np.all(y == 0.25)


# ---- GELU (exact erf form)
def test_gelu_known_values():
    # x * Phi(x) with textbook values of the normal CDF
    assert abs(O.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15
    assert abs(O.gelu(np.array([-1.0]))[0] + 0.15865525393145707) < 1e-15
    assert abs(O.gelu(np.array([2.0]))[0] - 2 * 0.9772498680518208) < 1e-15
    assert O.gelu(np.array([0.0]))[0] == 0.0


def test_gelu_identities_and_torch():
    x = np.linspace(-8, 8, 4001)
    y = O.gelu(x)
    assert np.allclose(y - O.gelu(-x), x, atol=1e-14)          # odd part is x/2 * 2
    assert np.allclose(y[x > 7], x[x > 7], atol=1e-10)         # -> x
    assert np.abs(y[x < -7]).max() < 1e-10                     # -> 0
    want = F.gelu(torch.from_numpy(x), approximate="none").numpy()
    assert np.allclose(y, want, atol=1e-14)
    # the tanh approximation is a different function: make sure we are not it
    tanh_form = F.gelu(torch.from_numpy(x), approximate="tanh").numpy()
    assert np.abs(y - tanh_form).max() > 1e-4


# ---- log-softmax and top-k
def test_log_softmax_normalised_and_torch():
    rng = np.random.default_rng(4)
    l = rng.standard_normal((6, 333)) * 5 + 100.0              # large offset: stable form needed
    logp, lse = O.log_softmax(l)
    assert np.allclose(np.exp(logp).sum(-1), 1.0, atol=1e-12)
    want = torch.log_softmax(torch.from_numpy(l), -1).numpy()
    assert np.allclose(logp, want, atol=1e-12)
    assert np.allclose(lse, torch.logsumexp(torch.from_numpy(l), -1).numpy(), atol=1e-12)


def test_topk_desc_order_and_ties():
    v = np.array([1.0, 5.0, 3.0, 5.0, -2.0, 3.0, 5.0])
    assert O.topk_desc(v, 5).tolist() == [1, 3, 6, 2, 5]       # equal values: smaller index first
    rng = np.random.default_rng(5)
    x = rng.standard_normal(1000)
    got = O.topk_desc(x, 7)
    want = torch.topk(torch.from_numpy(x), 7).indices.numpy()
    assert got.tolist() == want.tolist()


# ---- one stage against torch building blocks (non-square so a transpose shows)
def _tiny_weights(rng, n, E, D, V, affine=True):
    w = {"proj": [], "emb": [], "head": [], "ln_gamma": [], "ln_beta": []}
    for i in range(n):
        w["proj"].append(rng.standard_normal((D, E if i == 0 else D)) * 0.3)
        w["emb"].append(rng.standard_normal((V, D)) * 0.7)
        w["head"].append(rng.standard_normal((V, D)) * 0.5)
        w["ln_gamma"].append(1 + 0.2 * rng.standard_normal(D) if affine else np.ones(D))
        w["ln_beta"].append(0.2 * rng.standard_normal(D) if affine else np.zeros(D))
    return w


def test_single_stage_matches_torch_modules():
    rng = np.random.default_rng(6)
    E, D, V = 24, 16, 11
    w = _tiny_weights(rng, 1, E, D, V)
    s0 = rng.standard_normal((3, E))
    tok = np.array([4, 0, 10])
    w_s, w_e = 0.8, 0.6
    # oracle
    pz = O.project(s0, w["proj"][0])
    s = O.stage_state(pz, w["emb"][0][tok], w["ln_gamma"][0], w["ln_beta"][0], w_s, w_e, 1e-5, "f32")
    logp, _ = O.log_softmax(O.head_logits(s, w["head"][0]))
    # torch modules
    lin = torch.nn.Linear(E, D, bias=False, dtype=torch.float64)
    lin.weight.data = torch.from_numpy(w["proj"][0])
    emb = torch.nn.Embedding(V, D, dtype=torch.float64)
    emb.weight.data = torch.from_numpy(w["emb"][0])
    ln = torch.nn.LayerNorm(D, eps=1e-5, dtype=torch.float64)
    ln.weight.data = torch.from_numpy(w["ln_gamma"][0])
    ln.bias.data = torch.from_numpy(w["ln_beta"][0])
    head = torch.nn.Linear(D, V, bias=False, dtype=torch.float64)
    head.weight.data = torch.from_numpy(w["head"][0])
    with torch.no_grad():
        st = torch.nn.GELU()(ln(w_s * lin(torch.from_numpy(s0)) + w_e * emb(torch.from_numpy(tok))))
        lp = torch.log_softmax(head(st), -1)
    assert np.allclose(s, st.numpy(), atol=1e-12)
    assert np.allclose(logp, lp.numpy(), atol=1e-12)


def test_stage_state_bf16_is_rounded_once_at_the_end():
    rng = np.random.default_rng(7)
    pz = rng.standard_normal((4, 32))
    e = rng.standard_normal((4, 32))
    g, b = np.ones(32), np.zeros(32)
    s32 = O.stage_state(pz, e, g, b, 0.9, 0.4, 1e-5, "f32")
    s16 = O.stage_state(pz, e, g, b, 0.9, 0.4, 1e-5, "bf16")
    assert np.array_equal(s16, O.round_bf16(s32))
    assert np.abs(s16 - s32).max() > 0          # it did round
    assert np.abs(s16 - s32).max() <= np.abs(s32).max() * 2.0 ** -8
