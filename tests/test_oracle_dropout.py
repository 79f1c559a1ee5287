"""Pins of the oracle's dropout (CPU only): the keep decisions against the published SplitMix64 sequence,
the keep rate, special cases, and finite differences with the masks held fixed."""
import os

import numpy as np
import pytest

from oracle import mslt_oracle as O
from paper_2011_13635_amd import synth
from test_oracle_pins import small_case

GOLDEN_FILE = os.path.join(os.path.dirname(__file__), "golden", "splitmix64_seed0.txt")


def published_sequence():
    return [int(line, 16) for line in open(GOLDEN_FILE) if line.strip() and not line.startswith("#")]


def test_mix_reproduces_the_published_splitmix64_sequence():
    want = published_sequence()
    state, got = 0, []
    for _ in want:
        state = (state + O.GOLDEN) & ((1 << 64) - 1)
        got.append(O.mix64(state))
    assert got == want
    states = (np.arange(1, len(want) + 1, dtype=np.uint64) * np.uint64(O.GOLDEN))
    assert [int(v) for v in O.mix64_array(states)] == want


def test_mask_fields_follow_the_documented_layout():
    # element e is decided by bits 16*(e%4) .. +15 of mix64(key + (e//4) * GOLDEN); recomputed here with Python ints
    d = O.Dropout(0.1, seed=12345, step=7)
    shape = (5, 7)                       # 35 elements: a ragged last quad
    m = d.mask(3, O.SITE_FFN_OUT, shape).reshape(-1)
    key = O.dropout_key(12345, 7, 3, O.SITE_FFN_OUT)
    for e in range(35):
        r = O.mix64(key + (e // 4) * O.GOLDEN)
        keep = ((r >> (16 * (e % 4))) & 0xFFFF) >= 6554
        assert m[e] == (1.0 / 0.9 if keep else 0.0)
    assert d.thr == 6554
    # different step, layer or site: a different mask
    same = d.mask(3, O.SITE_FFN_OUT, shape)
    assert np.array_equal(same.reshape(-1), m)
    for other in (O.Dropout(0.1, 12345, 8).mask(3, O.SITE_FFN_OUT, shape), d.mask(2, O.SITE_FFN_OUT, shape),
                  d.mask(3, O.SITE_ATTN_OUT, shape), O.Dropout(0.1, 12346, 7).mask(3, O.SITE_FFN_OUT, shape)):
        assert not np.array_equal(other, same)


def test_keep_rate_and_scale():
    d = O.Dropout(0.1, seed=1, step=0)
    m = d.mask(0, O.SITE_ATTN_PROBS, (4, 2, 64, 64))
    kept = np.count_nonzero(m) / m.size
    assert abs(kept - 0.9) < 4 * np.sqrt(0.09 / m.size)          # binomial, four sigma
    assert set(np.unique(m)) == {0.0, 1.0 / 0.9}
    assert abs(m.mean() - 1.0) < 5e-3                            # unbiased in expectation
    for field in range(4):                                       # each 16-bit field on its own
        assert abs(np.count_nonzero(m.reshape(-1)[field::4]) / (m.size / 4) - 0.9) < 0.01


def test_p_zero_changes_nothing_and_p_changes_the_loss():
    sh, W, batch = small_case()
    l0, g0, _ = O.stage_step(sh, W, batch, 1, 1)
    l1, g1, _ = O.stage_step(sh, W, batch, 1, 1, drop=O.Dropout(0.0, 9, 3))
    assert l0 == l1 and all(np.array_equal(g0[k], g1[k]) for k in g0)
    l2, _, _ = O.stage_step(sh, W, batch, 1, 1, drop=O.Dropout(0.1, 9, 3))
    assert abs(l2 - l0) > 1e-6


def test_frozen_prefix_sees_dropout_too():
    # the output of the frozen prefix changes with the step number (its masks change), not with what trains above
    sh, W, batch = small_case()
    a = O.stage_step(sh, W, batch, 1, 1, drop=O.Dropout(0.1, 9, 3))[2]["prefix_out"]
    b = O.stage_step(sh, W, batch, 1, 1, drop=O.Dropout(0.1, 9, 4))[2]["prefix_out"]
    c = O.forward(sh, W, batch, n_layers=1, drop=O.Dropout(0.1, 9, 3))[1]["XL"]
    assert not np.array_equal(a, b)
    assert np.array_equal(a, c)


@pytest.mark.parametrize("planted", [None, "attn", "ffn", "emb", "out"])
def test_finite_differences_with_fixed_masks(planted, monkeypatch):
    """With the masks fixed (same seed and step) the loss is a smooth function of the weights, so central
    differences pin the backward through every dropout site; a mask dropped from one backward site must fail."""
    sh, W, batch = small_case(ragged=True)
    W = {k: v.astype(np.float64) for k, v in W.items()}
    drop = O.Dropout(0.25, seed=5, step=2)    # a high rate so that every site matters
    if planted is not None:
        site = {"attn": O.SITE_ATTN_PROBS, "ffn": O.SITE_FFN_OUT, "emb": O.SITE_EMBEDDING, "out": O.SITE_ATTN_OUT}[planted]
        key = {"attn": "mA", "ffn": "mF", "emb": "mE", "out": "mO"}[planted]
        real_forward = O.forward

        def forward_then_forget(*a, **k):     # the backward no longer sees this site's mask
            loss, cache = real_forward(*a, **k)
            for c in cache["layers"]:
                if c is not None and key in c:
                    c[key] = None
            if key in cache["emb"]:
                cache["emb"][key] = None
            return loss, cache
        monkeypatch.setattr(O, "forward", forward_then_forget)
    loss, grads, _ = O.stage_step(sh, W, batch, 0, sh.n_layers, train_embeddings=True, full_backprop=True, drop=drop)
    if planted is not None:
        monkeypatch.undo()
    h = 1e-5
    rng = np.random.RandomState(1)
    bad = 0
    for name in W:
        big = np.abs(grads[name]).max()
        for c in rng.randint(0, W[name].size, size=3):
            if name == "emb.pos":
                c = c % (batch["input_ids"].shape[1] * sh.hidden)
            Wp, Wm = dict(W), dict(W)
            a = W[name].copy().ravel(); a[c] += h; Wp[name] = a.reshape(W[name].shape)
            a = W[name].copy().ravel(); a[c] -= h; Wm[name] = a.reshape(W[name].shape)
            fd = (O.forward(sh, Wp, batch, drop=drop)[0] - O.forward(sh, Wm, batch, drop=drop)[0]) / (2 * h)
            if abs(fd - grads[name].ravel()[c]) > 2e-6 * big + 1e-9:
                bad += 1
    if planted is None:
        assert bad == 0
    else:
        assert bad > 0, f"a backward without the {planted} mask went unnoticed"
