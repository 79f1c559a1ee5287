"""GPU parity with dropout on (Section 4.1: the settings of BERT): the keep decisions are counter-based, so the
oracle reproduces every mask bit for bit and losses and gradients are compared at the usual tolerances."""
import numpy as np
import pytest

from paper_2011_13635_amd import binding, synth
from parity_util import assert_parity, grads_dict, make_model, run_case
from test_parity_gpu import small_shape

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("precision", [0, 1])
@pytest.mark.parametrize("f,k,emb", [(0, 3, True), (1, 2, False), (2, 1, False)])
def test_tiny_with_dropout(precision, f, k, emb):
    # tiny BERT: every site (embedding, attention probabilities, attention output, FFN output), frozen and
    # trainable layers, dense lower layers and the compacted top layer
    sh = synth.tiny_shape()
    std, perturb = (0.08, 0.1) if precision == 0 else (0.02, 0.05)
    r = run_case(sh, 3, 40, f, k, emb, precision, ragged=True, seed=3, std=std, perturb=perturb, dropout=(0.1, 77, 5))
    print("dropout tiny", precision, f, k, emb, assert_parity(r, precision, f"dropout tiny {f}/{k}"))
    r["model"].close()


@pytest.mark.parametrize("precision", [0, 1])
def test_unaligned_with_dropout(precision):
    # guarded kernels (wave-per-row attention, SIMT products), a high rate
    sh = small_shape(2)
    std, perturb = (0.2, 0.2) if precision == 0 else (0.05, 0.05)
    r = run_case(sh, 11, 13, 0, 2, True, precision, ragged=True, seed=5, std=std, perturb=perturb, dropout=(0.25, 3, 0))
    print("dropout unaligned", precision, assert_parity(r, precision, "dropout unaligned"))
    r["model"].close()


def test_base_one_tile_and_long_sequences_with_dropout():
    # BERT-Base width in bf16: S = 128 takes the one-launch attention backward, S = 256 the two-kernel one
    sh = synth.bert_base_shape(3)
    for B, S, f, k in ((4, 128, 1, 2), (2, 256, 1, 2)):
        r = run_case(sh, B, S, f, k, False, 1, ragged=True, seed=11, std=0.02, perturb=0.05, dropout=(0.1, 2024, 123456))
        print("dropout base", B, S, assert_parity(r, 1, f"dropout base {B}x{S}"))
        r["model"].close()


def test_masks_repeat_with_the_step_number_and_only_then():
    sh = synth.tiny_shape()
    W = synth.make_weights(sh, 1)
    m = make_model(sh, 4, 64, 0)
    m.mslt_load_params(synth.pack_weights(sh, W))
    cb = m.device_batch(synth.make_batch(sh, 4, 64, seed=2))
    base = m.mslt_stage_step(1, 2, False, cb)
    g_base = m.mslt_get_grads()
    m.mslt_set_dropout(0.1, 9, 4)
    a = m.mslt_stage_step(1, 2, False, cb)
    ga = m.mslt_get_grads()
    prefix_a = m.mslt_debug_prefix_output(4, 64)
    a2 = m.mslt_stage_step(1, 2, False, cb)
    assert a == a2 and np.array_equal(ga, m.mslt_get_grads())          # same (seed, step): same masks, bit for bit
    m.mslt_set_dropout(0.1, 9, 5)
    b = m.mslt_stage_step(1, 2, False, cb)
    assert b != a and a != base
    assert not np.array_equal(prefix_a, m.mslt_debug_prefix_output(4, 64))   # the frozen prefix is dropped too
    m.mslt_set_dropout(0.0, 9, 5)
    c = m.mslt_stage_step(1, 2, False, cb)
    assert c == base and np.array_equal(g_base, m.mslt_get_grads())   # p = 0: exactly the path without dropout
    with pytest.raises(binding.MsltError):
        m.mslt_set_dropout(1.0, 1, 1)
    m.close()
