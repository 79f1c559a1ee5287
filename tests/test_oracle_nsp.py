"""Pins of the oracle's next-sentence head (pooler + two-way classifier, the second objective of BERT that
Section 4.1 keeps), CPU only: closed forms, finite differences, and that it reaches the encoder only through the
first token of every sequence."""
import math

import numpy as np

from oracle import mslt_oracle as O
from paper_2011_13635_amd import synth


def nsp_case(seed=3, n_layers=2):
    sh = synth.ModelShape(n_layers=n_layers, hidden=32, n_heads=2, ffn=64, vocab=50, max_pos=16, nsp=True)
    W = {k: v.astype(np.float64) for k, v in synth.make_weights(sh, seed=seed, std=0.25, perturb=0.2).items()}
    batch = synth.make_batch(sh, 4, 10, seed=seed + 1, ragged=True)
    return sh, W, batch


def test_names_and_labels():
    sh, W, batch = nsp_case()
    assert [n for n in W][-4:] == ["pooler.w", "pooler.b", "nsp.w", "nsp.b"]
    assert W["nsp.w"].shape == (2, 32) and W["pooler.w"].shape == (32, 32)
    assert batch["nsp_labels"].shape == (4,) and set(np.unique(batch["nsp_labels"])) <= {0, 1}
    assert synth.trainable_names(sh, 1, 1, False)[-4:] == list(O.NSP_TENSORS)
    assert O.decays("pooler.w") and O.decays("nsp.w") and not O.decays("pooler.b") and not O.decays("nsp.b")


def test_zero_classifier_gives_ln2_and_the_mlm_loss_is_added():
    sh, W, batch = nsp_case()
    plain = synth.ModelShape(n_layers=2, hidden=32, n_heads=2, ffn=64, vocab=50, max_pos=16)
    mlm = O.forward(plain, {k: v for k, v in W.items() if k.split(".")[0] not in ("pooler", "nsp")}, batch)[0]
    W0 = dict(W)
    W0["nsp.w"] = np.zeros_like(W["nsp.w"]); W0["nsp.b"] = np.zeros_like(W["nsp.b"])
    total, grads, _ = O.stage_step(sh, W0, batch, 0, 2, True)
    assert abs(total - (mlm + math.log(2.0))) < 1e-12
    # with a zero classifier: d nsp.b = mean(softmax - onehot) = [0.5 - frac(label 0), 0.5 - frac(label 1)]
    y = batch["nsp_labels"]
    want = np.array([0.5 - np.mean(y == 0), 0.5 - np.mean(y == 1)])
    assert np.allclose(grads["nsp.b"], want, atol=1e-15)
    assert np.abs(grads["pooler.w"]).max() == 0.0          # nothing flows back through a zero classifier


def test_finite_differences_with_the_second_objective():
    sh, W, batch = nsp_case()
    loss, grads, _ = O.stage_step(sh, W, batch, 0, 2, True, full_backprop=True)
    assert set(grads) == set(W)
    h, rng, bad = 1e-5, np.random.RandomState(4), []
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


def test_classifier_sees_only_the_first_token_rows():
    # pooler and classifier gradients depend on the last layer's output only through rows b*S
    sh, W, batch = nsp_case()
    _, cache = O.forward(sh, W, batch)
    ops = O.Ops()
    dXc, g = O.nsp_backward(sh, cache["P64"], cache["nsp"], ops)
    assert dXc.shape == (4, 32)
    assert list(cache["nsp"]["cls"]) == [0, 10, 20, 30]
    XL2 = cache["XL"].copy()
    keep = np.zeros(len(XL2), dtype=bool); keep[cache["nsp"]["cls"]] = True
    XL2[~keep] += 1.0                                       # perturb every other row
    l2, _ = O.nsp_forward(sh, cache["P64"], XL2, 4, 10, np.asarray(batch["nsp_labels"], dtype=np.int64), ops)
    l1, _ = O.nsp_forward(sh, cache["P64"], cache["XL"], 4, 10, np.asarray(batch["nsp_labels"], dtype=np.int64), ops)
    assert l1 == l2
