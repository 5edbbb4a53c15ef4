"""GPU parity at the full sizes of the build's five configurations, in the launch
configuration the benchmark times.  Inputs are drawn on the device (the CPU
generator needs minutes for 10^9 normals) and copied to the host for the oracle.
The oracle compares EVERY sequence of the 7B- and 13B-shaped batches; of the
70B-class batch (2.6 TFLOP of float64 head rows per step) it compares 16 of the 32
sequences (sequences are independent); the verify properties that hold for any
input are checked on all of them."""
import pytest

from paper_2404_19124_amd import workloads as W
from tests.gpu_common import run_workload

pytestmark = pytest.mark.gpu


def _exempt_allowance(rows: int) -> int:
    """Rows whose tokens may differ from the oracle's own (each one validated inside the strict band on the
    same state): a bf16 flip of the state moves logits by up to ~5e-3, and about one row in a hundred has
    two of its best logits that close."""
    return max(2, rows // 100)


def test_llama7b_batch1():
    rep, *_ = run_workload(W.WORKLOADS["llama7b_b1"])
    assert rep.rows_checked + rep.rows_skipped_below_exempt == 21
    assert rep.rows_exempt <= 1


def test_llama7b_batch1_other_seed_with_affine():
    wl = W.small_variant(W.WORKLOADS["llama7b_b1"], seed=7, emb_std=0.2)
    rep, *_ = run_workload(wl, ln_affine="random")
    assert rep.rows_exempt <= 1


def test_llama7b_batch64():
    wl = W.WORKLOADS["llama7b_b64"]
    rep, *_ = run_workload(wl)                      # all 64 sequences
    assert rep.seqs == 64 and rep.rows_checked + rep.rows_skipped_below_exempt == sum(wl.rows()) == 1344
    assert rep.rows_exempt <= _exempt_allowance(1344)


def test_llama13b_batch16():
    wl = W.WORKLOADS["llama13b_b16"]
    rep, *_ = run_workload(wl)                      # all 16 sequences
    assert rep.seqs == 16 and rep.rows_checked + rep.rows_skipped_below_exempt == sum(wl.rows()) == 496
    assert rep.rows_exempt <= _exempt_allowance(496)


def test_large70b_batch32_sampled():
    wl = W.WORKLOADS["large70b_b32"]
    seqs = list(range(0, 32, 2))                    # 16 of the 32 sequences
    rep, *_ = run_workload(wl, sample_seqs=seqs)
    assert rep.seqs == 16 and rep.rows_checked + rep.rows_skipped_below_exempt == 16 * (1 + 6 + 24 + 72)
    assert rep.rows_exempt <= _exempt_allowance(16 * 103)


# ---- code-model shapes: 7 and 5 heads, k = 1 chains and a small tree (Sec. 4.3, 4.4)

def test_code13b_seven_heads_chain_batch1():
    wl = W.WORKLOADS["code13b_k1_b1"]
    rep, step, od, _ = run_workload(wl)
    assert rep.rows_checked + rep.rows_skipped_below_exempt == 7
    assert rep.rows_exempt <= 1
    assert step.cand_tokens.shape == (1, 1, 7)


def test_code13b_seven_heads_small_tree_batch4():
    rep, *_ = run_workload(W.WORKLOADS["code13b_tree_b4"], ln_affine="random")
    assert rep.rows_exempt <= 2


def test_code20b_five_heads_chain_batch8():
    rep, *_ = run_workload(W.WORKLOADS["code20b_k1_b8"])
    assert rep.rows_exempt <= 1
