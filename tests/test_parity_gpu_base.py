"""GPU parity at BERT-Base shapes (bf16 mode with fp32 master weights): a reduced batch the oracle
finishes in seconds, and the full benchmark configuration (6 layers present, bottom 3 frozen, top
3 trainable, batch 64 x seq 128) compared against the oracle on every gradient element."""
import numpy as np
import pytest

from paper_2011_13635_amd import synth
from parity_util import assert_parity, run_case

pytestmark = pytest.mark.gpu


def test_base_stage2_reduced_batch():
    sh = synth.bert_base_shape(6)
    r = run_case(sh, 8, 128, 3, 3, False, 1, full_backprop=False)
    print("base 3/3 8x128", assert_parity(r, 1, "base-reduced"))
    r["model"].close()


def test_base_ragged_long_sequence():
    sh = synth.bert_base_shape(2)
    r = run_case(sh, 3, 200, 1, 1, False, 1, ragged=True, seed=7, full_backprop=False)
    print("base 1/1 3x200 ragged", assert_parity(r, 1, "base-ragged"))
    r["model"].close()


def test_base_full_step_with_embeddings():
    sh = synth.bert_base_shape(2)
    r = run_case(sh, 8, 128, 0, 2, True, 1, seed=2, full_backprop=False)
    print("base 0/2+emb 8x128", assert_parity(r, 1, "base-full"))
    r["model"].close()


def test_base_stage2_benchmark_configuration():
    sh = synth.bert_base_shape(6)
    r = run_case(sh, 64, 128, 3, 3, False, 1, full_backprop=False)
    print("base 3/3 64x128", assert_parity(r, 1, "base-bench"))
    assert len(r["pos"]) == 64 * 19
    r["model"].close()
