"""GPU parity at BERT-Base shapes (bf16 mode with fp32 master weights): a reduced batch the oracle
finishes in seconds, and the full benchmark configuration (6 layers present, bottom 3 frozen, top
3 trainable, batch 64 x seq 128) compared against the oracle on every gradient element."""
import numpy as np
import pytest

from paper_2011_13635_amd import synth
from parity_util import TOL, assert_parity, run_case

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
    r = run_case(sh, 64, 128, 3, 3, False, 1, full_backprop=False, rounded_oracle=True)
    print("base 3/3 64x128", assert_parity(r, 1, "base-bench"))
    assert len(r["pos"]) == 64 * 19
    r["model"].close()


def test_base_final_stage_long_sequence():
    # final stage of the Base schedule at sequence length 512 (attention tiled over keys), reduced batch
    sh = synth.bert_base_shape(4)
    r = run_case(sh, 2, 512, 3, 1, False, 1, seed=3, full_backprop=False)
    print("base 3/1 2x512", assert_parity(r, 1, "base-512"))
    r["model"].close()


def test_large_stage_with_lamb_update():
    # BERT-Large shapes (hidden 1024, 16 heads, FFN 4096), 1 frozen + 2 trainable layers, LAMB update
    import numpy as np
    from oracle import mslt_oracle as O
    from paper_2011_13635_amd import binding
    sh = synth.bert_large_shape(3)
    r = run_case(sh, 8, 128, 1, 2, False, 1, seed=4, full_backprop=False)
    print("large 1/2 8x128", assert_parity(r, 1, "large"))
    m = r["model"]
    before = synth.unpack_weights(sh, m.mslt_get_params())
    opt = binding.lamb(lr=0.00088)
    m.mslt_apply_update(opt)
    after = synth.unpack_weights(sh, m.mslt_get_params())
    trainable = set(synth.trainable_names(sh, 1, 2, False))
    W64 = O.to_f64({n: r["W"][n] for n in trainable})
    st = O.new_opt_state(W64)
    new_ref, ratios = O.optimizer_update(W64, r["ref_grads"], st, kind="lamb", lr=0.00088)
    for name in before:
        if name not in trainable:
            assert np.array_equal(before[name], after[name]), name
            continue
        dw = after[name].astype(np.float64) - before[name].astype(np.float64)
        if name.endswith(".bk"):
            continue
        wn = np.linalg.norm(before[name].astype(np.float64))
        if wn > 0:   # LAMB: the step of every tensor with a non-zero norm has length lr*|w|
            assert abs(np.linalg.norm(dw) - 0.00088 * wn) < 2e-3 * 0.00088 * wn, name
        # (the element-wise update is compared in fp32 mode in test_parity_gpu.py; in bf16 mode the adaptive
        #  direction g/(|g|+eps) turns gradient noise of small entries into sign flips, so only the direction
        #  as a whole is compared here)
        dref = new_ref[name] - W64[name]
        cos = float((dw * dref).sum() / (np.linalg.norm(dw) * np.linalg.norm(dref) + 1e-300))
        assert cos > 0.8, (name, cos)
    m.close()


def test_base_final_stage_full_size():
    # final stage of the BERT-Base schedule at full size: 12 layers, bottom 9 frozen, top 3 trainable,
    # batch 64 x seq 128; every gradient element against the oracle
    sh = synth.bert_base_shape(12)
    r = run_case(sh, 64, 128, 9, 3, False, 1, perturb=0.05, full_backprop=False, rounded_oracle=True)
    print("base 9/3 64x128", assert_parity(r, 1, "base-final"))
    r["model"].close()


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_large_final_stage_full_size(seed):
    # final stage of the BERT-Large schedule at full size: 24 layers, bottom 18 frozen, top 6 trainable,
    # batch 64 x seq 128, on three seeds.  Two references on every seed.  The sharp one is the oracle on the
    # matrices as bf16 mode reads them (the fp32 masters rounded to bf16 where they feed the matrix cores): what
    # is left is the kernels' own arithmetic, asserted at 1.2e-2.  The other is the oracle on the fp32 masters:
    # rounding the matrices alone already moves the query/key gradients of the lowest trainable layer by 1.3e-2
    # to 1.7e-2 of their largest entry (oracle against oracle), so the two parts together scatter around 2e-2
    # from seed to seed (measured 1.4e-2 to 2.0e-2, always a W_k of a low trainable layer; 0.5e-2 to 0.6e-2 against
    # the rounded matrices); that comparison is asserted at
    # 3e-2 for the gradients and at 2e-2 for the loss and the frozen-prefix output.
    sh = synth.bert_large_shape(24)
    r = run_case(sh, 64, 128, 18, 6, False, 1, seed=seed, perturb=0.05 if seed == 2 else 0.0, full_backprop=False,
                 rounded_oracle=True)
    print("large 18/6 64x128 seed", seed, assert_parity(r, 1, "large-final", grad_tol=1.5 * TOL[1]))
    if seed == 0:
        # the LAMB update of this step (Section 4.1: LAMB, learning rate 0.00088), element by element: the oracle's
        # optimizer on the library's own fp32 gradients
        from oracle import mslt_oracle as O
        from paper_2011_13635_amd import binding
        m = r["model"]
        names = synth.trainable_names(sh, 18, 6, False)
        before = synth.unpack_weights(sh, m.mslt_get_params())
        m.mslt_apply_update(binding.lamb(lr=0.00088))
        after = synth.unpack_weights(sh, m.mslt_get_params())
        W64 = O.to_f64({n: before[n] for n in names})
        new_ref, _ = O.optimizer_update(W64, {n: r["grads"][n] for n in names}, O.new_opt_state(W64), kind="lamb", lr=0.00088)
        for n in before:
            if n not in names:
                assert np.array_equal(before[n], after[n]), n
                continue
            dw, dref = after[n].astype(np.float64) - W64[n], new_ref[n] - W64[n]
            assert np.abs(dw - dref).max() <= 2e-4 * np.abs(dref).max() + 2.0 ** -22 * np.abs(W64[n]).max(), n
    r["model"].close()


def test_base_final_stage_full_size_long_sequences():
    # final stage of the BERT-Base schedule on the long sequences of the last tenth of training (Section 4.2):
    # 12 layers, bottom 9 frozen, top 3 trainable, batch 16 x seq 512; every gradient element against the oracle
    sh = synth.bert_base_shape(12)
    r = run_case(sh, 16, 512, 9, 3, False, 1, seed=5, perturb=0.05, full_backprop=False)
    print("base 9/3 16x512", assert_parity(r, 1, "base-final-long"))
    r["model"].close()


def test_large_sweep_size_top_layer_against_oracle_and_stage_equals_slice_of_full_step():
    # BERT-Large, 24 layers, batch 32 x seq 512 (the size of the schedule sweep).  The oracle needs minutes for
    # a six-layer backward at this size, so it checks the step that trains the top layer alone (all 24 layers
    # forward, one backward), and the six-layer stage is checked through the property that defines the method
    # (Section 3.2): its gradients are the same tensors' gradients of the step that trains all 24 layers.
    from parity_util import grads_dict, make_model
    sh = synth.bert_large_shape(24)
    r = run_case(sh, 32, 512, 23, 1, False, 1, seed=6, full_backprop=False)
    print("large 23/1 32x512", assert_parity(r, 1, "large-sweep-top"))
    m, cb = r["model"], r["cb"]
    ls = m.mslt_stage_step(18, 6, False, cb)
    gs = grads_dict(m, sh, 18, 6, False)
    ps = m.mslt_debug_prefix_output(32, 512)
    lf = m.mslt_stage_step(0, 24, False, cb)
    gf = grads_dict(m, sh, 0, 24, False)
    assert ls == lf, (ls, lf)
    assert abs(ls - r["ref_loss"]) < 1e-3 * abs(r["ref_loss"])       # the forward pass is that of the checked step
    worst = 0.0
    for name, g in gs.items():
        d = np.abs(g - gf[name]).max() / max(np.abs(gf[name]).max(), 1e-30)
        worst = max(worst, d)
        assert d <= 1e-6, (name, d)
    print("large 18/6 vs 0/24 32x512: worst relative difference", worst)
    assert np.isfinite(ps).all()
    m.close()


def test_two_stream_schedule_gives_the_single_stream_result_bit_for_bit():
    # The step spreads its kernels over two streams (the halves of the batch go through the encoder forward as two
    # chains; weight-gradient products run beside the data-gradient chain).  With per-kernel event timing switched
    # on everything runs on one stream in program order.  Both must give the same bits.
    from parity_util import make_model
    sh = synth.bert_base_shape(4)
    m = make_model(sh, 8, 128, 1)
    m.mslt_load_params(synth.pack_weights(sh, synth.make_weights(sh, seed=8)))
    cb = m.device_batch(synth.make_batch(sh, 8, 128, seed=9))
    for p in (0.0, 0.1):       # with dropout the second half's kernels must take the decisions of their own positions
        m.mslt_set_dropout(p, 77, 3)
        l2 = m.mslt_stage_step(2, 2, False, cb)
        g2 = m.mslt_get_grads().copy()
        m.mslt_profile_enable(True)
        l1 = m.mslt_stage_step(2, 2, False, cb)
        g1 = m.mslt_get_grads().copy()
        m.mslt_profile_enable(False)
        assert l1 == l2, p
        assert np.array_equal(g1, g2), p
    m.close()


def test_a_run_of_training_steps_on_two_streams_gives_the_single_stream_result_bit_for_bit():
    # A run of steps (layer split changing in between, growth, then a step that trains everything) must leave the
    # same parameters whether the kernels are spread over the two streams or all run on one in program order.
    from paper_2011_13635_amd import binding
    from parity_util import make_model
    sh = synth.bert_base_shape(4)
    W = synth.pack_weights(sh, synth.make_weights(sh, seed=11))
    batches = [synth.make_batch(sh, 8, 128, seed=20 + i) for i in range(6)]
    results = []
    for serial in (False, True):
        m = make_model(sh, 8, 128, 1)
        m.mslt_load_params(W)
        m.mslt_profile_enable(serial)
        cbs = [m.device_batch(b) for b in batches]
        losses = []
        losses.append(m.mslt_train_step(0, 2, True, cbs[0], binding.lamb(lr=1e-3)))
        losses.append(m.mslt_train_step(0, 2, True, cbs[1], binding.lamb(lr=1e-3)))
        m.mslt_grow(2, 2)
        losses.append(m.mslt_train_step(2, 2, False, cbs[2], binding.lamb(lr=1e-3)))
        losses.append(m.mslt_train_step(2, 2, False, cbs[3], binding.adam(lr=1e-4)))
        losses.append(m.mslt_train_step(3, 1, False, cbs[4], binding.adam(lr=1e-4)))   # layer 2 was just updated
        losses.append(m.mslt_train_step(0, 4, True, cbs[5], binding.adam(lr=1e-4)))
        results.append((losses, m.mslt_get_params().copy()))
        m.close()
    assert results[0][0] == results[1][0]
    assert np.array_equal(results[0][1], results[1][1])


def test_benchmark_configuration_training_run_is_reproducible_bit_for_bit():
    # ten training steps of the benchmark configuration, twice from the same weights and once more on one
    # stream: the kernels of a step overlap on two streams in an order that varies from run to run, and none
    # of that may show in the result
    from paper_2011_13635_amd import binding
    from parity_util import make_model
    sh = synth.bert_base_shape(6)
    W = synth.pack_weights(sh, synth.make_weights(sh, seed=0))
    batches = [synth.make_batch(sh, 64, 128, seed=1 + i) for i in range(2)]
    out = []
    for serial in (False, False, True):
        m = make_model(sh, 64, 128, 1)
        m.mslt_load_params(W)
        m.mslt_profile_enable(serial)
        cbs = [m.device_batch(b) for b in batches]
        losses = [m.mslt_train_step(3, 3, False, cbs[i % 2], binding.adam(lr=1e-4)) for i in range(10)]
        out.append((losses, m.mslt_get_params().copy()))
        m.close()
    for other in out[1:]:
        assert other[0] == out[0][0]
        assert np.array_equal(other[1], out[0][1])
