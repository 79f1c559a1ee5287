"""GPU parity of the grouped variant (Section 3.3: the layers of a group share one parameter set and the
gradients of a set add up over its applications), against the oracle."""
import numpy as np
import pytest

from oracle import mslt_oracle as O
from paper_2011_13635_amd import binding, synth
from parity_util import assert_parity, make_model, run_case

pytestmark = pytest.mark.gpu


def grouped_tiny(n_layers=4, g=2):
    return synth.ModelShape(n_layers=n_layers, hidden=128, n_heads=2, ffn=512, vocab=1024, max_pos=512, layers_per_group=g)


@pytest.mark.parametrize("precision", [0, 1])
@pytest.mark.parametrize("f,k,emb", [(0, 4, True), (2, 2, False), (0, 2, True)])
def test_grouped_tiny(precision, f, k, emb):
    sh = grouped_tiny()
    std, perturb = (0.08, 0.1) if precision == 0 else (0.02, 0.05)
    r = run_case(sh, 3, 40, f, k, emb, precision, ragged=True, seed=3, std=std, perturb=perturb)
    print("grouped tiny", precision, f, k, emb, assert_parity(r, precision, f"grouped {f}/{k}"))
    r["model"].close()


def test_grouped_three_per_group_with_dropout_bf16_base_width():
    # BERT-Base width, 6 layers in 2 groups of 3, the top group trained, dropout on: MFMA paths with accumulation
    sh = synth.ModelShape(n_layers=6, hidden=768, n_heads=12, ffn=3072, vocab=30522, layers_per_group=3)
    r = run_case(sh, 4, 128, 3, 3, False, 1, ragged=True, seed=11, std=0.02, perturb=0.05, dropout=(0.1, 5, 9))
    print("grouped base", assert_parity(r, 1, "grouped base 3/3"))
    r["model"].close()


def test_grouped_schedule_update_and_growth():
    # stage 1 trains group 0 (+ embeddings), growth copies it into group 1, stage 2 trains group 1 only
    sh = grouped_tiny()
    W = synth.make_weights(sh, 4)
    m = make_model(sh, 4, 64, 0)
    m.mslt_load_params(synth.pack_weights(sh, W))
    ref = O.to_f64(W)
    st = O.new_opt_state(ref)
    opt = binding.adam(lr=0.002)
    E = binding
    cb = m.device_batch(synth.make_batch(sh, 4, 64, seed=10))
    assert m.mslt_stage_step(1, 2, False, cb, allow=(E.MSLT_ERR_ARG,)) == E.MSLT_ERR_ARG     # not whole groups
    for step in range(2):
        batch = synth.make_batch(sh, 4, 64, seed=10 + step)
        loss = m.mslt_train_step(0, 2, True, m.device_batch(batch), opt)
        rl, rg, _ = O.stage_step(sh, ref, batch, 0, 2, True)
        ref, _ = O.optimizer_update(ref, rg, st, kind="adam", lr=0.002)
        assert abs(loss - rl) / rl < 1e-4
    m.mslt_grow(2, 2)
    ref = O.grow(ref, 1, 1)
    for t in O.LAYER_TENSORS:
        st[f"layer1.{t}"] = {"m": np.zeros_like(ref[f"layer1.{t}"]), "v": np.zeros_like(ref[f"layer1.{t}"]), "t": 0}
    frozen_before = synth.unpack_weights(sh, m.mslt_get_params())
    for t in O.LAYER_TENSORS:
        assert np.array_equal(frozen_before[f"layer1.{t}"], frozen_before[f"layer0.{t}"])
    for step in range(2):
        batch = synth.make_batch(sh, 4, 64, seed=20 + step)
        loss = m.mslt_train_step(2, 2, False, m.device_batch(batch), opt)
        rl, rg, _ = O.stage_step(sh, ref, batch, 2, 2, False)
        ref, _ = O.optimizer_update(ref, rg, st, kind="adam", lr=0.002)
        assert abs(loss - rl) / rl < 1e-4, (step, loss, rl)
    got = synth.unpack_weights(sh, m.mslt_get_params())
    for t in O.LAYER_TENSORS:                      # the frozen group is bit-unchanged
        assert np.array_equal(got[f"layer0.{t}"], frozen_before[f"layer0.{t}"])
    for name in got:
        d = np.abs(got[name] - ref[name]).max()
        assert d < 2e-3 * max(np.abs(ref[name]).max(), 1e-3), (name, d)
    m.close()
