"""The update entry point that allocates nothing (its scratch is a device array inside the library)
against mslt_apply_update: same parameters bit for bit, on two calls in a row, the second one on a
smaller set of trainable tensors."""
import numpy as np
import pytest

from paper_2011_13635_amd import binding, synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("precision", [0, 1])
def test_static_scratch_update_equals_workspace_update(precision):
    shape = synth.ModelShape(n_layers=3, hidden=128, n_heads=2, ffn=512, vocab=1024, max_pos=64)
    W = synth.make_weights(shape, seed=0, perturb=0.05)
    flat = synth.pack_weights(shape, W)
    cfg = binding.make_config(shape, 4, 64, precision)
    ref = binding.Model(cfg, device="cuda:0")
    new = binding.Model(cfg, device="cuda:0")
    ref.mslt_load_params(flat)
    new.mslt_load_params(flat)
    opt = binding.lamb(lr=1e-3)
    # first call: everything trains (embeddings, 3 layers, head); second call: one layer and the head
    for i, (f, k, emb) in enumerate(((0, 3, True), (2, 1, False))):
        batch = synth.make_batch(shape, 4, 64, seed=1 + i, ragged=bool(i))
        l_ref = ref.mslt_stage_step(f, k, emb, ref.device_batch(batch))
        l_new = new.mslt_stage_step(f, k, emb, new.device_batch(batch))
        assert l_ref == l_new
        ref.mslt_apply_update(opt)
        ref.mslt_sync()
        new.mslt_apply_update_static(opt)
        new.mslt_sync()
        a, b = ref.mslt_get_params(), new.mslt_get_params()
        assert np.array_equal(a, b), f"call {i}: {np.abs(a - b).max()}"
        assert not np.array_equal(a, flat)
    # Adam through the same entry point (uses no scratch at all)
    batch = synth.make_batch(shape, 4, 64, seed=5)
    ref.mslt_stage_step(1, 2, False, ref.device_batch(batch))
    new.mslt_stage_step(1, 2, False, new.device_batch(batch))
    ref.mslt_apply_update(binding.adam())
    new.mslt_apply_update_static(binding.adam())
    assert np.array_equal(ref.mslt_get_params(), new.mslt_get_params())
    # call order errors are those of the existing entry point
    with pytest.raises(binding.MsltError) as ei:
        new.mslt_apply_update_static(opt)
    assert ei.value.code == binding.MSLT_ERR_STATE
    ref.close()
    new.close()
