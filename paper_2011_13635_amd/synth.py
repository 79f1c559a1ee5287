"""Seeded synthetic inputs for an MSLT stage step: model shapes, weights, token batches.

This module holds no arithmetic of the training method itself (no encoder, loss,
gradient or optimizer code).  It only produces the inputs that both the CPU oracle
and the HIP library consume: the tensor list of a BERT stack with a masked-LM head,
initial weights, and token/mask/label batches that stand in for the paper's
Wikipedia+BookCorpus pre-training data (Section 4.1), which is not available.

Randomness is a counter-based 64-bit integer mixer keyed by (seed, stream, index),
so every value is a pure function of its key and does not depend on numpy's
generator implementation.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict
import numpy as np

# synthetic vocabulary: reserved ids, ordinary ids start at 4
PAD_ID, CLS_ID, SEP_ID, MASK_ID, FIRST_ORDINARY_ID = 0, 1, 2, 3, 4
IGNORE_LABEL = -100

# stream identifiers of the counter-based generator
_STREAM_WEIGHTS, _STREAM_TOKENS, _STREAM_LENGTHS, _STREAM_MASKPOS, _STREAM_MASKKIND, _STREAM_MASKRAND = (
    11, 12, 13, 14, 15, 16)
_STREAM_NSP = 17


@dataclass(frozen=True)
class ModelShape:
    """Shape of a BERT encoder stack with a tied masked-LM head (BERT by citation, Section 4.1)."""
    n_layers: int
    hidden: int
    n_heads: int
    ffn: int
    vocab: int
    max_pos: int = 512
    type_vocab: int = 2
    ln_eps: float = 1e-12
    mask_bias: float = -10000.0
    # grouped ALBERT variant (Section 3.3): runs of this many consecutive layers share one parameter set,
    # named layer{g}.* for group g; 1 = every layer has its own set (BERT)
    layers_per_group: int = 1
    # next-sentence head (Section 4.1 keeps BERT's second objective): pooler (dense + tanh on the first
    # token) and a two-way classifier, tensors pooler.w, pooler.b, nsp.w, nsp.b after the masked-LM head
    nsp: bool = False

    @property
    def n_param_sets(self):
        return self.n_layers // self.layers_per_group

    def as_dict(self):
        return asdict(self)


# Shapes the paper's commented-out hyper-parameter table gives (Section 4.1), plus the tiny test model.
def tiny_shape(n_layers=3):
    return ModelShape(n_layers=n_layers, hidden=128, n_heads=2, ffn=512, vocab=1024, max_pos=512)


def bert_base_shape(n_layers=12):
    return ModelShape(n_layers=n_layers, hidden=768, n_heads=12, ffn=3072, vocab=30522)


def bert_large_shape(n_layers=24):
    return ModelShape(n_layers=n_layers, hidden=1024, n_heads=16, ffn=4096, vocab=30522)


LAYER_TENSORS = ("wq", "wk", "wv", "bq", "bk", "bv", "wo", "bo", "ln1_g", "ln1_b",
                 "w1", "b1", "w2", "b2", "ln2_g", "ln2_b")


def tensor_specs(shape: ModelShape):
    """Canonical tensor list: (name, shape tuple, kind) with kind in matrix/bias/gamma/beta.

    Order: embedding block, encoder layers bottom to top, masked-LM head.  Weight
    matrices are [out, in] row-major.
    """
    H, F, V = shape.hidden, shape.ffn, shape.vocab
    specs = [
        ("emb.word", (V, H), "matrix"),
        ("emb.pos", (shape.max_pos, H), "matrix"),
        ("emb.type", (shape.type_vocab, H), "matrix"),
        ("emb.ln_g", (H,), "gamma"),
        ("emb.ln_b", (H,), "beta"),
    ]
    for i in range(shape.n_param_sets):
        p = f"layer{i}."
        specs += [
            (p + "wq", (H, H), "matrix"), (p + "wk", (H, H), "matrix"), (p + "wv", (H, H), "matrix"),
            (p + "bq", (H,), "bias"), (p + "bk", (H,), "bias"), (p + "bv", (H,), "bias"),
            (p + "wo", (H, H), "matrix"), (p + "bo", (H,), "bias"),
            (p + "ln1_g", (H,), "gamma"), (p + "ln1_b", (H,), "beta"),
            (p + "w1", (F, H), "matrix"), (p + "b1", (F,), "bias"),
            (p + "w2", (H, F), "matrix"), (p + "b2", (H,), "bias"),
            (p + "ln2_g", (H,), "gamma"), (p + "ln2_b", (H,), "beta"),
        ]
    specs += [
        ("head.wt", (H, H), "matrix"), ("head.bt", (H,), "bias"),
        ("head.ln_g", (H,), "gamma"), ("head.ln_b", (H,), "beta"),
        ("head.b_out", (V,), "bias"),
    ]
    if shape.nsp:
        specs += [("pooler.w", (H, H), "matrix"), ("pooler.b", (H,), "bias"),
                  ("nsp.w", (2, H), "matrix"), ("nsp.b", (2,), "bias")]
    return specs


# ----------------------------------------------------------------------------------------------
# counter-based generator
# ----------------------------------------------------------------------------------------------
_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix64(x):
    """Finalising 64-bit integer mixer (add the golden-ratio increment, two xor-shift-multiply rounds)."""
    x = np.asarray(x, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = x + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def rand_u64(seed: int, stream: int, index):
    """64 random bits for each entry of `index`, a pure function of (seed, stream, index)."""
    k = _mix64(np.uint64(seed & 0xFFFFFFFFFFFFFFFF))
    k = _mix64(k ^ np.uint64(stream))
    return _mix64(k ^ np.asarray(index, dtype=np.uint64))


def rand_uniform(seed: int, stream: int, index):
    """Uniform deviates strictly inside (0, 1), 53 bits."""
    z = rand_u64(seed, stream, index)
    return ((z >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def rand_normal(seed: int, stream: int, start: int, n: int):
    """n standard normal deviates (Box-Muller on uniform pairs 2i, 2i+1 of the stream)."""
    out = np.empty(n, dtype=np.float64)
    step = 1 << 22
    for s in range(0, n, step):
        e = min(n, s + step)
        idx = np.arange(start + s, start + e, dtype=np.uint64)
        u1 = rand_uniform(seed, stream, idx * np.uint64(2))
        u2 = rand_uniform(seed, stream, idx * np.uint64(2) + np.uint64(1))
        out[s:e] = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return out


# ----------------------------------------------------------------------------------------------
# weights
# ----------------------------------------------------------------------------------------------
def make_weights(shape: ModelShape, seed: int = 0, std: float = 0.02, perturb: float = 0.0):
    """Initial weights as float32 arrays keyed by tensor name.

    Default recipe: matrices and embeddings N(0, std) (not truncated), biases 0,
    LayerNorm gamma 1 and beta 0.  With perturb > 0 (test-only variety) biases and
    beta get N(0, perturb) and gamma gets 1 + N(0, perturb), so that tests are
    sensitive to every term of the backward pass.
    """
    out = {}
    start = 0
    for name, shp, kind in tensor_specs(shape):
        n = int(np.prod(shp))
        if kind == "matrix":
            w = std * rand_normal(seed, _STREAM_WEIGHTS, start, n)
        elif kind == "gamma":
            w = np.ones(n) + (perturb * rand_normal(seed, _STREAM_WEIGHTS, start, n) if perturb else 0.0)
        else:
            w = perturb * rand_normal(seed, _STREAM_WEIGHTS, start, n) if perturb else np.zeros(n)
        out[name] = np.ascontiguousarray(w.reshape(shp).astype(np.float32))
        start += n
    return out


def pack_weights(shape: ModelShape, weights) -> np.ndarray:
    """Concatenate a name->array dict into one float32 vector in canonical tensor order."""
    return np.concatenate([np.asarray(weights[n], dtype=np.float32).ravel() for n, _, _ in tensor_specs(shape)])


def unpack_weights(shape: ModelShape, flat, names=None):
    """Split a flat vector holding the tensors `names` (default: all) back into a dict."""
    specs = {n: s for n, s, _ in tensor_specs(shape)}
    order = [n for n, _, _ in tensor_specs(shape)] if names is None else list(names)
    out, o = {}, 0
    for n in order:
        cnt = int(np.prod(specs[n]))
        out[n] = np.asarray(flat[o:o + cnt]).reshape(specs[n])
        o += cnt
    assert o == len(flat), (o, len(flat))
    return out


def trainable_names(shape: ModelShape, frozen_layers: int, trainable_layers: int, train_embeddings: bool):
    """Names of the tensors one stage step produces gradients for, in canonical order.

    Section 3.2: the newly added top layers and the output layer train; the embedding
    block (with the tied word matrix) trains only when nothing below is frozen.
    """
    names = []
    if train_embeddings:
        names += ["emb.word", "emb.pos", "emb.type", "emb.ln_g", "emb.ln_b"]
    g = shape.layers_per_group
    for i in range(frozen_layers // g, (frozen_layers + trainable_layers) // g):
        names += [f"layer{i}.{t}" for t in LAYER_TENSORS]
    names += ["head.wt", "head.bt", "head.ln_g", "head.ln_b", "head.b_out"]
    if shape.nsp:
        names += ["pooler.w", "pooler.b", "nsp.w", "nsp.b"]
    return names


# ----------------------------------------------------------------------------------------------
# token batches
# ----------------------------------------------------------------------------------------------
def zipf_cdf(n_ranks: int, s: float = 1.1) -> np.ndarray:
    w = np.arange(1, n_ranks + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(w)
    return c / c[-1]


def n_masked_for_length(length: int) -> int:
    """Number of predicted positions of a sequence with `length` non-pad tokens (15 %, at least one)."""
    cand = length - 2
    return max(1, int(np.floor(0.15 * cand + 0.5)))


def make_batch(shape: ModelShape, batch: int, seq: int, seed: int = 1, ragged: bool = False):
    """One masked-LM batch.

    Returns int32 arrays input_ids, token_type_ids, attn_mask, labels of shape
    [batch, seq] and the flat ascending list of predicted positions.
      * ordinary token ids follow a truncated Zipf(1.1) over ranks 1..V-4, rank r -> id 3+r;
      * position 0 is CLS, the last valid position is SEP, another SEP sits at len//2;
        token type is 0 up to and including that middle SEP and 1 after it;
      * ragged=True draws each length uniformly from [seq//2, seq], else every sequence is full;
      * 15 % of the positions strictly between the first and last valid token are
        chosen by a seeded partial shuffle; of those 80 % become MASK, 10 % a uniformly
        random ordinary id, 10 % stay; labels hold the original id there and -100 elsewhere.
    """
    V = shape.vocab
    assert seq >= 4 and seq <= shape.max_pos and V > FIRST_ORDINARY_ID + 1
    cdf = zipf_cdf(V - FIRST_ORDINARY_ID)
    idx = np.arange(batch * seq, dtype=np.uint64)
    u = rand_uniform(seed, _STREAM_TOKENS, idx)
    ranks = np.minimum(np.searchsorted(cdf, u, side="left"), V - FIRST_ORDINARY_ID - 1) + 1
    ids = (ranks + (FIRST_ORDINARY_ID - 1)).astype(np.int64).reshape(batch, seq)

    if ragged:
        ul = rand_uniform(seed, _STREAM_LENGTHS, np.arange(batch, dtype=np.uint64))
        lo = max(4, seq // 2)
        lengths = lo + np.floor(ul * (seq - lo + 1)).astype(np.int64)
        lengths = np.minimum(lengths, seq)
    else:
        lengths = np.full(batch, seq, dtype=np.int64)

    token_type = np.zeros((batch, seq), dtype=np.int64)
    attn_mask = np.zeros((batch, seq), dtype=np.int64)
    labels = np.full((batch, seq), IGNORE_LABEL, dtype=np.int64)
    for b in range(batch):
        L = int(lengths[b])
        ids[b, 0] = CLS_ID
        ids[b, L - 1] = SEP_ID
        mid = L // 2
        ids[b, mid] = SEP_ID
        ids[b, L:] = PAD_ID
        token_type[b, mid + 1:L] = 1
        attn_mask[b, :L] = 1
        # partial Fisher-Yates shuffle over candidate positions 1..L-2
        cand = np.arange(1, L - 1, dtype=np.int64)
        m = n_masked_for_length(L)
        m = min(m, len(cand))
        ush = rand_uniform(seed, _STREAM_MASKPOS, np.uint64(b) * np.uint64(1 << 20) + np.arange(m, dtype=np.uint64))
        for j in range(m):
            k = j + int(np.floor(ush[j] * (len(cand) - j)))
            cand[j], cand[k] = cand[k], cand[j]
        chosen = np.sort(cand[:m])
        key = np.uint64(b) * np.uint64(1 << 20) + chosen.astype(np.uint64)
        uk = rand_uniform(seed, _STREAM_MASKKIND, key)
        ur = rand_uniform(seed, _STREAM_MASKRAND, key)
        for p, a, r in zip(chosen, uk, ur):
            labels[b, p] = ids[b, p]
            if a < 0.8:
                ids[b, p] = MASK_ID
            elif a < 0.9:
                ids[b, p] = FIRST_ORDINARY_ID + int(np.floor(r * (V - FIRST_ORDINARY_ID)))
    flat_pos = np.flatnonzero(labels.ravel() != IGNORE_LABEL).astype(np.int32)
    return {
        "input_ids": ids.astype(np.int32),
        "token_type_ids": token_type.astype(np.int32),
        "attn_mask": attn_mask.astype(np.int32),
        "labels": labels.astype(np.int32),
        "masked_positions": flat_pos,
        "lengths": lengths.astype(np.int32),
        # next-sentence label of each sequence (1 = the second segment is a random one), a seeded coin
        "nsp_labels": (rand_uniform(seed, _STREAM_NSP, np.arange(batch, dtype=np.uint64)) < 0.5).astype(np.int32),
    }
