"""Pins of the CPU oracle against things other than itself: finite differences, literal
triple-loop products, closed forms, invariants and special cases (no GPU)."""
import math

import numpy as np
import pytest

from oracle import mslt_oracle as O
from paper_2011_13635_amd import synth


def small_shape(n_layers=2):
    return synth.ModelShape(n_layers=n_layers, hidden=32, n_heads=2, ffn=64, vocab=50, max_pos=16)


def small_case(n_layers=2, ragged=True, seed=3, std=0.25, perturb=0.2, B=3, S=10):
    sh = small_shape(n_layers)
    W = synth.make_weights(sh, seed=seed, std=std, perturb=perturb)
    batch = synth.make_batch(sh, B, S, seed=seed + 1, ragged=ragged)
    return sh, W, batch


def loss_only(sh, W, batch, n=None):
    return O.forward(sh, W, batch, n_layers=n)[0]


def fd_check(ragged, coords_per_tensor=4):
    """Largest |finite difference - analytic| excess over the tolerance, over sampled coordinates of every tensor."""
    sh, W, batch = small_case(ragged=ragged)
    W = {k: v.astype(np.float64) for k, v in W.items()}
    loss, grads, _ = O.stage_step(sh, W, batch, 0, sh.n_layers, train_embeddings=True, full_backprop=True)
    assert set(grads) == set(W)
    h = 1e-5
    rng = np.random.RandomState(0)
    used_ids = np.unique(batch["input_ids"])
    failures = []
    for name in W:
        n = W[name].size
        coords = set(rng.randint(0, n, size=coords_per_tensor).tolist())
        if name == "emb.word":   # rows that are looked up get both tied contributions
            coords |= {int(used_ids[1]) * sh.hidden + 3, int(batch["labels"].max()) * sh.hidden + 5}
        if name == "emb.pos":
            coords = {c % (batch["input_ids"].shape[1] * sh.hidden) for c in coords}
        big = np.abs(grads[name]).max()
        for c in coords:
            Wp = dict(W); Wm = dict(W)
            a = W[name].copy().ravel(); a[c] += h; Wp[name] = a.reshape(W[name].shape)
            a = W[name].copy().ravel(); a[c] -= h; Wm[name] = a.reshape(W[name].shape)
            fd = (loss_only(sh, Wp, batch) - loss_only(sh, Wm, batch)) / (2 * h)
            an = grads[name].ravel()[c]
            # absolute floor 1e-9: rounding of the two loss values divided by 2h; the key bias has a
            # mathematically zero gradient (softmax is shift-invariant) and only sees that floor
            if abs(fd - an) > 2e-6 * big + 1e-9:
                failures.append((name, c, fd, an))
            if name.endswith(".bk"):
                assert abs(an) < 1e-12
    return failures


@pytest.mark.parametrize("ragged", [False, True])
def test_finite_differences_every_tensor(ragged):
    assert fd_check(ragged) == []


def test_finite_differences_catch_planted_mistakes(monkeypatch):
    """Each plausible slip in the oracle's backward (planted here, on the CPU) must trip the check."""
    good_gelu_grad, good_ln_bwd = O.gelu_grad, O.layer_norm_backward

    def gelu_grad_no_pdf(u):          # dropped term u*phi(u)
        return 0.5 * (1.0 + O._erf(u / math.sqrt(2.0)))

    def ln_bwd_no_mean(dy, g, cache):  # dropped mean-subtraction term
        xhat, rstd = cache
        dxh = dy * g
        dz = (dxh - xhat * (dxh * xhat).mean(axis=-1, keepdims=True)) * rstd
        return dz, (dy * xhat).sum(axis=0), dy.sum(axis=0)

    def ln_bwd_no_gamma(dy, g, cache):  # forgot gamma on the way down
        dz, dg, db = good_ln_bwd(dy, np.ones_like(g), cache)
        return dz, dg, db

    for attr, bad in (("gelu_grad", gelu_grad_no_pdf), ("layer_norm_backward", ln_bwd_no_mean),
                      ("layer_norm_backward", ln_bwd_no_gamma)):
        monkeypatch.setattr(O, attr, bad)
        assert fd_check(False, coords_per_tensor=2) != [], attr
        monkeypatch.undo()
    assert O.gelu_grad is good_gelu_grad and fd_check(False, coords_per_tensor=1) == []


def test_triple_loop_products_agree_with_blas():
    sh = synth.ModelShape(n_layers=1, hidden=8, n_heads=2, ffn=12, vocab=20, max_pos=8)
    W = synth.make_weights(sh, seed=1, std=0.3, perturb=0.2)
    batch = synth.make_batch(sh, 2, 5, seed=2, ragged=True)
    l1, g1, _ = O.stage_step(sh, W, batch, 0, 1, True, ops=O.Ops(naive=False), full_backprop=True)
    l2, g2, _ = O.stage_step(sh, W, batch, 0, 1, True, ops=O.Ops(naive=True), full_backprop=True)
    assert abs(l1 - l2) < 1e-12
    for k in g1:
        assert np.abs(g1[k] - g2[k]).max() <= 1e-12 * max(1.0, np.abs(g1[k]).max()), k


def test_softmax_and_layernorm_invariants():
    sh, W, batch = small_case()
    loss, cache = O.forward(sh, W, batch)
    for c in cache["layers"]:
        assert np.allclose(c["P"].sum(-1), 1.0, atol=1e-13)
        assert (c["P"] >= 0).all()
    # padded keys get (numerically) no probability
    am = batch["attn_mask"]
    for b in range(am.shape[0]):
        pad = np.flatnonzero(am[b] == 0)
        if len(pad):
            assert cache["layers"][0]["P"][b][:, :, pad].max() < 1e-300
    rng = np.random.RandomState(1)
    z = rng.randn(7, 33) * 3 + 1
    y, (xh, rstd) = O.layer_norm(z, np.ones(33), np.zeros(33), 1e-12)
    assert np.allclose(y.mean(-1), 0, atol=1e-14)
    var = z.var(-1)
    assert np.allclose(y.var(-1), var / (var + 1e-12), rtol=1e-12)
    # textbook values for one row: z = (1,2,3,4): mean 2.5, biased var 1.25
    y, _ = O.layer_norm(np.array([[1.0, 2, 3, 4]]), np.array([2.0, 2, 2, 2]), np.array([1.0, 1, 1, 1]), 0.0)
    assert np.allclose(y, 1 + 2 * np.array([-1.5, -0.5, 0.5, 1.5]) / math.sqrt(1.25))
    # where epsilon sits: a two-element row (-1e-6, +1e-6) has mean 0 and biased variance 1e-12, the size of BERT's
    # epsilon itself (BERT by citation, Section 4.1), so with epsilon added to the variance under the root the
    # normalised values are -+1/sqrt(2); added to the standard deviation instead they would be -+1 (to 1e-6), with
    # no epsilon exactly -+1, and with the unbiased variance -+1/sqrt(3)
    y, _ = O.layer_norm(np.array([[-1e-6, 1e-6]]), np.ones(2), np.zeros(2), 1e-12)
    assert np.allclose(y, [[-math.sqrt(0.5), math.sqrt(0.5)]], rtol=1e-12)
    # ... and the model configurations carry that epsilon
    assert synth.tiny_shape(1).ln_eps == 1e-12 and synth.bert_large_shape(24).ln_eps == 1e-12
    # backward invariants
    dy = rng.randn(7, 33)
    g = rng.randn(33)
    _, cache_ln = O.layer_norm(z, g, np.zeros(33), 1e-12)
    dz, dg, db = O.layer_norm_backward(dy, g, cache_ln)
    assert np.allclose(dz.sum(-1), 0, atol=1e-12)
    assert np.allclose((dz * cache_ln[0]).sum(-1), 0, atol=1e-12)
    assert np.allclose(db, dy.sum(0))


def test_gelu_values_and_slope():
    # Phi(1) = 0.841344746..., so gelu(1) = 0.8413447; gelu(0)=0, gelu'(0)=1/2
    assert abs(O.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15
    assert O.gelu(np.array([0.0]))[0] == 0.0
    assert abs(O.gelu_grad(np.array([0.0]))[0] - 0.5) < 1e-16
    x = np.linspace(-4, 4, 41)
    fd = (O.gelu(x + 1e-6) - O.gelu(x - 1e-6)) / 2e-6
    assert np.abs(fd - O.gelu_grad(x)).max() < 1e-9
    assert np.all(np.abs(O.gelu(x) - np.maximum(x, 0)) < 0.2)


def test_loss_closed_form_ln_vocab():
    # with the head LayerNorm's gamma = beta = 0 and zero output bias every logit is 0:
    # loss = ln V exactly and dZ = (1/V - onehot)/M
    for V in (50, 1024):
        sh = synth.ModelShape(n_layers=1, hidden=32, n_heads=2, ffn=64, vocab=V, max_pos=16)
        W = synth.make_weights(sh, seed=0, std=0.1)
        W["head.ln_g"][:] = 0
        batch = synth.make_batch(sh, 3, 12, seed=1)
        loss, grads, info = O.stage_step(sh, W, batch, 0, 1, True, full_backprop=True)
        assert abs(loss - math.log(V)) < 1e-13
        M = len(info["pos"])
        cnt = np.bincount(info["labels"], minlength=V)
        assert np.allclose(grads["head.b_out"], (M / V - cnt) / M, atol=1e-15)
    assert abs(math.log(1024) - 6.931472) < 1e-6 and abs(math.log(30522) - 10.326203) < 1e-6
    # N(0, 0.02) initialisation stays close to ln V
    sh = synth.tiny_shape()
    loss = O.forward(sh, synth.make_weights(sh, 0), synth.make_batch(sh, 4, 64, 1))[0]
    assert abs(loss - math.log(1024)) < 5e-2


def test_rows_of_dlogits_sum_to_zero_and_dA_rows():
    sh, W, batch = small_case()
    loss, cache = O.forward(sh, W, batch)
    P = cache["P64"]
    _, _, _, dZ = O.head_backward(sh, P, cache["head"], cache["T"], O.Ops())
    assert np.allclose(dZ.sum(-1), 0, atol=1e-15)
    assert np.allclose(dZ.sum(), 0, atol=1e-14)


def test_attention_special_cases():
    # zero query projection -> uniform attention over unpadded keys -> context = mean of value rows
    sh, W, batch = small_case(n_layers=1)
    W["layer0.wq"][:] = 0
    W["layer0.bq"][:] = 0
    loss, cache = O.forward(sh, W, batch)
    c = cache["layers"][0]
    B, S = batch["input_ids"].shape
    for b in range(B):
        L = int(batch["lengths"][b])
        mean_v = c["V"][b * S:b * S + L].mean(axis=0)
        assert np.allclose(c["C"][b * S:(b + 1) * S], mean_v[None, :], atol=1e-12)
    # a single key: P == 1 and the layer is an MLP of X -> V -> out
    sh1 = synth.ModelShape(n_layers=1, hidden=8, n_heads=2, ffn=12, vocab=20, max_pos=8)
    W1 = O.to_f64(synth.make_weights(sh1, seed=1, std=0.3, perturb=0.2))
    X = np.random.RandomState(0).randn(3, 8)
    X2, c1 = O.layer_forward(sh1, W1, 0, X, np.zeros((3, 1)), 3, 1, O.Ops())
    assert np.all(c1["P"] == 1.0)
    Vv = X @ W1["layer0.wv"].T + W1["layer0.bv"]
    assert np.allclose(c1["C"], Vv)
    x1, _ = O.layer_norm(X + Vv @ W1["layer0.wo"].T + W1["layer0.bo"], W1["layer0.ln1_g"], W1["layer0.ln1_b"], sh1.ln_eps)
    x2, _ = O.layer_norm(x1 + O.gelu(x1 @ W1["layer0.w1"].T + W1["layer0.b1"]) @ W1["layer0.w2"].T + W1["layer0.b2"],
                         W1["layer0.ln2_g"], W1["layer0.ln2_b"], sh1.ln_eps)
    assert np.allclose(X2, x2, atol=1e-13)


def test_attention_score_scale_two_keys_by_hand():
    # BERT's scaled dot-product attention (Section 4.1 takes the network by citation): scores are
    # q.k / sqrt(d_h).  One head of width 4, two keys, identity query/key projections, all numbers
    # typed out: q1 = k1 = (1, 2, 0, -1), q2 = k2 = (0.5, -1, 3, 2).
    sh = synth.ModelShape(n_layers=1, hidden=4, n_heads=1, ffn=8, vocab=20, max_pos=8)
    W = O.to_f64(synth.make_weights(sh, seed=5, std=0.3, perturb=0.1))
    W["layer0.wq"] = np.eye(4)
    W["layer0.wk"] = np.eye(4)
    W["layer0.bq"] = np.zeros(4)
    W["layer0.bk"] = np.zeros(4)
    X = np.array([[1.0, 2.0, 0.0, -1.0], [0.5, -1.0, 3.0, 2.0]])
    _, c = O.layer_forward(sh, W, 0, X, np.zeros((1, 2)), 1, 2, O.Ops())
    # dot products: q1.k1 = 6, q1.k2 = q2.k1 = -3.5, q2.k2 = 14.25; d_h = 4, so they are halved
    s11, s12, s22 = 6.0 / 2.0, -3.5 / 2.0, 14.25 / 2.0
    p11 = 1.0 / (1.0 + math.exp(s12 - s11))
    p22 = 1.0 / (1.0 + math.exp(s12 - s22))
    want = np.array([[p11, 1.0 - p11], [1.0 - p22, p22]])
    assert np.allclose(c["P"][0, 0], want, rtol=0, atol=1e-14)
    # the unscaled scores and a division by d_h instead of its root give visibly different rows
    for wrong in (1.0, 0.25):
        q11 = 1.0 / (1.0 + math.exp(wrong * (-3.5 - 6.0)))
        assert abs(q11 - c["P"][0, 0, 0, 0]) > 1e-4
    # and the context is that mixture of the two value rows
    V = X @ W["layer0.wv"].T + W["layer0.bv"]
    assert np.allclose(c["C"], want @ V, atol=1e-13)


def test_stage_step_equals_slice_of_full_step():
    # Section 3.1/3.2: the trainable tensors get the gradients plain back-propagation gives them;
    # the frozen prefix only supplies the input of the top layers.
    sh, W, batch = small_case(n_layers=4, B=2, S=8)
    l_full, g_full, i_full = O.stage_step(sh, W, batch, 0, 4, True, full_backprop=True)
    for f, k in ((2, 2), (3, 1), (1, 3)):
        l, g, info = O.stage_step(sh, W, batch, f, k, False)
        l2, g2, info2 = O.stage_step(sh, W, batch, f, k, False, full_backprop=True)
        assert l == l_full and l2 == l_full
        assert set(g) == set(synth.trainable_names(sh, f, k, False))
        for name in g:
            assert np.array_equal(g[name], g_full[name]), name
            assert np.array_equal(g2[name], g_full[name]), name
        assert "emb.word" not in g and f"layer{f - 1}.wq" not in g
    # prefix output independent of what trains above it, and equal to a forward-only run of the prefix
    _, _, a = O.stage_step(sh, W, batch, 2, 1, False)
    _, _, b = O.stage_step(sh, W, batch, 2, 2, False)
    assert np.array_equal(a["prefix_out"], b["prefix_out"])
    _, cache2 = O.forward(sh, W, batch, n_layers=2)
    assert np.array_equal(cache2["XL"], a["prefix_out"])
    # fewer layers present -> a different model: the loss changes
    assert O.stage_step(sh, W, batch, 2, 1, False)[0] != l_full
    with pytest.raises(ValueError):
        O.stage_step(sh, W, batch, 1, 1, True)
    with pytest.raises(ValueError):
        O.stage_step(sh, W, batch, 3, 2, False)


def test_update_touches_only_trainable_tensors():
    sh, W, batch = small_case(n_layers=3, B=2, S=8)
    W64 = O.to_f64(W)
    state = O.new_opt_state(W64)
    _, g, _ = O.stage_step(sh, W, batch, 2, 1, False)
    for kind in ("adam", "lamb"):
        st = O.new_opt_state(W64)
        new, _ = O.optimizer_update(W64, g, st, kind=kind, lr=1e-3)
        for name in W64:
            if name in g:
                assert not np.array_equal(new[name], W64[name]) or np.abs(g[name]).max() == 0, name
                assert st[name]["t"] == 1
            else:
                assert np.array_equal(new[name], W64[name]), name   # bit-unchanged, tied word matrix included
                assert st[name]["t"] == 0 and not st[name]["m"].any()
    assert "emb.word" not in g


def test_adam_closed_forms():
    rng = np.random.RandomState(0)
    w = {"layer0.w1": rng.randn(5, 4), "layer0.b1": rng.randn(5)}
    g = {"layer0.w1": rng.randn(5, 4), "layer0.b1": rng.randn(5)}
    lr, eps = 1e-3, 1e-6
    st = O.new_opt_state(w)
    new, _ = O.optimizer_update(w, g, st, "adam", lr=lr, eps=eps, weight_decay=0.0, bias_correction=True)
    for k in w:   # first step from zero state: -lr g / (|g| + eps)
        assert np.allclose(new[k] - w[k], -lr * g[k] / (np.abs(g[k]) + eps), rtol=1e-9, atol=0)
    st = O.new_opt_state(w)
    new, _ = O.optimizer_update(w, g, st, "adam", lr=lr, eps=eps, weight_decay=0.0, bias_correction=False)
    for k in w:
        assert np.allclose(new[k] - w[k], -lr * 0.1 * g[k] / (math.sqrt(0.001) * np.abs(g[k]) + eps), rtol=1e-9, atol=0)
    # decoupled decay acts on the matrix only
    st = O.new_opt_state(w)
    new, _ = O.optimizer_update(w, g, st, "adam", lr=lr, eps=eps, weight_decay=0.01)
    k = "layer0.w1"
    assert np.allclose(new[k] - w[k], -lr * (g[k] / (np.abs(g[k]) + eps) + 0.01 * w[k]), rtol=1e-9, atol=0)
    k = "layer0.b1"
    assert np.allclose(new[k] - w[k], -lr * g[k] / (np.abs(g[k]) + eps), rtol=1e-9, atol=0)
    # second step uses both moments: check against the recurrences typed out for one scalar
    w1 = {"head.bt": np.array([0.3])}
    st = O.new_opt_state(w1)
    a, _ = O.optimizer_update(w1, {"head.bt": np.array([2.0])}, st, "adam", lr=0.1, eps=0.0, weight_decay=0.0)
    b, _ = O.optimizer_update(a, {"head.bt": np.array([-1.0])}, st, "adam", lr=0.1, eps=0.0, weight_decay=0.0)
    m2 = 0.9 * 0.2 + 0.1 * -1.0
    v2 = 0.999 * 0.004 + 0.001 * 1.0
    exp = 0.3 - 0.1 - 0.1 * (m2 / (1 - 0.81)) / math.sqrt(v2 / (1 - 0.999 ** 2))
    assert abs(b["head.bt"][0] - exp) < 1e-12


def test_lamb_closed_forms():
    rng = np.random.RandomState(1)
    w = {"layer0.w1": rng.randn(6, 4), "layer0.b1": np.zeros(6), "layer0.wq": rng.randn(4, 4)}
    g = {k: rng.randn(*v.shape) for k, v in w.items()}
    lr = 0.00088
    st = O.new_opt_state(w)
    new, ratios = O.optimizer_update(w, g, st, "lamb", lr=lr, weight_decay=0.01)
    for k in ("layer0.w1", "layer0.wq"):   # |dw| = lr |w| for every tensor with a non-zero norm
        assert abs(np.linalg.norm(new[k] - w[k]) - lr * np.linalg.norm(w[k])) < 1e-12
    k = "layer0.b1"                       # zero tensor: ratio 1, plain step
    assert ratios[k] == 1.0
    assert np.allclose(new[k], -lr * g[k] / (np.abs(g[k]) + 1e-6), rtol=1e-9)


def test_masked_positions_match_generator():
    sh = synth.tiny_shape()
    for ragged in (False, True):
        batch = synth.make_batch(sh, 4, 64, seed=7, ragged=ragged)
        pos, Y = O.masked_rows(batch)
        assert np.array_equal(pos, batch["masked_positions"])
        assert (np.diff(pos) > 0).all()
        assert np.array_equal(Y, batch["labels"].ravel()[pos])
        assert (Y >= 0).all()


def test_grow_copies_top_layers_in_order():
    sh, W, _ = small_case(n_layers=4)
    W2 = O.grow(W, 2, 2)
    for t in O.LAYER_TENSORS:
        assert np.array_equal(W2[f"layer2.{t}"], W[f"layer0.{t}"])
        assert np.array_equal(W2[f"layer3.{t}"], W[f"layer1.{t}"])
        assert np.array_equal(W2[f"layer0.{t}"], W[f"layer0.{t}"])


def test_oracle_names_match_generator_names():
    sh = synth.tiny_shape()
    for f, k, e in ((0, 3, True), (2, 1, False), (1, 2, False)):
        assert O.stage_tensor_names(f, k, e) == synth.trainable_names(sh, f, k, e)
    for n, _, kind in synth.tensor_specs(sh):
        assert O.decays(n) == (kind == "matrix"), n
