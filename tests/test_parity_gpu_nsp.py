"""GPU parity with the next-sentence head (pooler + two-way classifier; Section 4.1 keeps both objectives of
BERT): loss = masked-LM loss + next-sentence loss, and the classifier's gradient reaches the encoder through the
first token of every sequence, which therefore joins the compacted rows of the top layer."""
import numpy as np
import pytest

from oracle import mslt_oracle as O
from paper_2011_13635_amd import binding, synth
from parity_util import assert_parity, make_model, run_case

pytestmark = pytest.mark.gpu


def nsp_tiny(n_layers=3, **kw):
    return synth.ModelShape(n_layers=n_layers, hidden=128, n_heads=2, ffn=512, vocab=1024, max_pos=512, nsp=True, **kw)


@pytest.mark.parametrize("precision", [0, 1])
@pytest.mark.parametrize("f,k,emb", [(0, 3, True), (1, 2, False), (2, 1, False)])
def test_tiny_with_next_sentence_head(precision, f, k, emb):
    sh = nsp_tiny()
    std, perturb = (0.08, 0.1) if precision == 0 else (0.02, 0.05)
    r = run_case(sh, 3, 40, f, k, emb, precision, ragged=True, seed=3, std=std, perturb=perturb)
    assert set(O.NSP_TENSORS) <= set(r["grads"])
    print("nsp tiny", precision, f, k, emb, assert_parity(r, precision, f"nsp tiny {f}/{k}"))
    r["model"].close()


def test_base_width_bf16_with_both_objectives_dropout_and_groups():
    sh = synth.ModelShape(n_layers=4, hidden=768, n_heads=12, ffn=3072, vocab=30522, nsp=True, layers_per_group=2)
    r = run_case(sh, 8, 128, 2, 2, False, 1, ragged=True, seed=13, std=0.02, perturb=0.05, dropout=(0.1, 8, 2))
    print("nsp base", assert_parity(r, 1, "nsp base 2/2"))
    r["model"].close()


def test_training_with_both_objectives_follows_the_oracle_and_rejects_bad_labels():
    sh = nsp_tiny(2)
    W = synth.make_weights(sh, 4)
    m = make_model(sh, 4, 64, 0)
    m.mslt_load_params(synth.pack_weights(sh, W))
    ref = O.to_f64(W)
    st = O.new_opt_state(ref)
    opt = binding.lamb(lr=0.002)
    for step in range(3):
        batch = synth.make_batch(sh, 4, 64, seed=40 + step, ragged=True)
        loss = m.mslt_train_step(1, 1, False, m.device_batch(batch), opt)
        rl, rg, _ = O.stage_step(sh, ref, batch, 1, 1, False)
        ref, _ = O.optimizer_update(ref, rg, st, kind="lamb", lr=0.002)
        assert abs(loss - rl) / rl < 1e-4, (step, loss, rl)
    got = synth.unpack_weights(sh, m.mslt_get_params())
    for name in got:
        d = np.abs(got[name] - ref[name]).max()
        assert d < 2e-3 * max(np.abs(ref[name]).max(), 1e-3), (name, d)
    for t in O.NSP_TENSORS:                                   # the second head trains in a later stage too
        assert not np.array_equal(got[t], W[t])
    E = binding
    bad = synth.make_batch(sh, 4, 64, seed=50)
    bad["nsp_labels"] = bad["nsp_labels"].copy(); bad["nsp_labels"][2] = 2
    assert m.mslt_stage_step(1, 1, False, m.device_batch(bad), allow=(E.MSLT_ERR_DATA,)) == E.MSLT_ERR_DATA
    nolab = synth.make_batch(sh, 4, 64, seed=50)
    del nolab["nsp_labels"]
    assert m.mslt_stage_step(1, 1, False, m.device_batch(nolab), allow=(E.MSLT_ERR_ARG,)) == E.MSLT_ERR_ARG
    m.close()
