"""Pins of the oracle's grouped-layer variant (Section 3.3: the layers of a group share one parameter set), CPU only:
against the ungrouped oracle on copied parameters (chain rule: a shared tensor's gradient is the sum over its uses)
and against finite differences."""
import numpy as np
import pytest

from oracle import mslt_oracle as O
from paper_2011_13635_amd import synth


def grouped_case(n_layers=4, g=2, seed=3):
    sh = synth.ModelShape(n_layers=n_layers, hidden=32, n_heads=2, ffn=64, vocab=50, max_pos=16, layers_per_group=g)
    W = {k: v.astype(np.float64) for k, v in synth.make_weights(sh, seed=seed, std=0.25, perturb=0.2).items()}
    batch = synth.make_batch(sh, 3, 10, seed=seed + 1, ragged=True)
    return sh, W, batch


def test_parameter_sets_and_names():
    sh, W, _ = grouped_case()
    assert sh.n_param_sets == 2
    assert {k.split(".")[0] for k in W if k.startswith("layer")} == {"layer0", "layer1"}
    assert synth.trainable_names(sh, 2, 2, False)[:1] == ["layer1.wq"]
    assert O.stage_tensor_names(2, 2, False, 2)[:1] == ["layer1.wq"]


def test_grouped_equals_ungrouped_with_copied_parameters():
    sh, W, batch = grouped_case()
    flat = synth.ModelShape(n_layers=4, hidden=32, n_heads=2, ffn=64, vocab=50, max_pos=16)
    Wflat = {k: v for k, v in W.items() if not k.startswith("layer")}
    for i in range(4):
        for t in O.LAYER_TENSORS:
            Wflat[f"layer{i}.{t}"] = W[f"layer{i // 2}.{t}"].copy()
    lg, gg, _ = O.stage_step(sh, W, batch, 0, 4, True, full_backprop=True)
    lf, gf, _ = O.stage_step(flat, Wflat, batch, 0, 4, True, full_backprop=True)
    assert lg == lf
    for t in O.LAYER_TENSORS:
        for s in range(2):
            want = gf[f"layer{2 * s}.{t}"] + gf[f"layer{2 * s + 1}.{t}"]
            assert np.allclose(gg[f"layer{s}.{t}"], want, rtol=1e-12, atol=1e-15), (s, t)
    for k in gg:
        if not k.startswith("layer"):
            assert np.array_equal(gg[k], gf[k]), k
    # a later stage: group 0 frozen, group 1 trained; its gradients are those of the full step
    l2, g2, _ = O.stage_step(sh, W, batch, 2, 2, False)
    assert l2 == lg and set(g2) == set(O.stage_tensor_names(2, 2, False, 2))
    for k in g2:
        assert np.array_equal(g2[k], gg[k]), k
    with pytest.raises(ValueError):
        O.stage_step(sh, W, batch, 1, 2, False)         # not whole groups


def test_finite_differences_grouped():
    sh, W, batch = grouped_case()
    loss, grads, _ = O.stage_step(sh, W, batch, 0, 4, True, full_backprop=True)
    h, rng, bad = 1e-5, np.random.RandomState(2), []
    for name in W:
        big = np.abs(grads[name]).max()
        for c in rng.randint(0, W[name].size, size=3):
            if name == "emb.pos":
                c = c % (batch["input_ids"].shape[1] * sh.hidden)
            Wp, Wm = dict(W), dict(W)
            a = W[name].copy().ravel(); a[c] += h; Wp[name] = a.reshape(W[name].shape)
            a = W[name].copy().ravel(); a[c] -= h; Wm[name] = a.reshape(W[name].shape)
            fd = (O.forward(sh, Wp, batch)[0] - O.forward(sh, Wm, batch)[0]) / (2 * h)
            if abs(fd - grads[name].ravel()[c]) > 2e-6 * big + 1e-9:
                bad.append((name, c, fd, grads[name].ravel()[c]))
    assert not bad, bad[:3]
