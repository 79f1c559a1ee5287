"""CPU oracle for one MSLT stage step (TEST INFRASTRUCTURE, not a product path).

Plain numpy float64 implementation of what a stage step of Multi-Stage Layerwise
Training computes (paper Section 3.2): a BERT encoder stack (BERT by citation,
Section 4.1) with a tied masked-LM head, ordinary reverse-mode differentiation of the
masked-LM loss, from which the gradients of the trainable tensors (the top layers
and the output layer; everything in the first stage / the retraining stage) are
kept, and a textbook Adam / LAMB update (Sections 4.1 and 5 name the optimizers).

The method is exact: a stage step yields, for the tensors it trains, the very
gradients plain back-propagation would give, and simply omits the others (Section
3.1, last paragraph).  So this file is the plain definition written out; nothing is
blocked, fused or reordered.  Matrix products go through one hook (`Ops.mm`) that is
either numpy's matmul or a pure-Python triple loop for tiny cross-checks.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
file.  It imports nothing from the GPU package and shares no code with it.

Pins (tests/test_oracle_*.py): central finite differences of every tensor;
triple-loop products; softmax/LayerNorm invariants; loss = ln V closed form;
uniform-attention and S=1 special cases; stage-step gradients equal the full-step
gradients of the same tensors; Adam and LAMB one-step closed forms; dropout: the
generator against the published SplitMix64 sequence, keep rate, and finite
differences with the masks held fixed.  The paper
prints no worked numerical example, so absolute values have no published pin.
"""
from __future__ import annotations

import math
import numpy as np

LAYER_TENSORS = ("wq", "wk", "wv", "bq", "bk", "bv", "wo", "bo", "ln1_g", "ln1_b",
                 "w1", "b1", "w2", "b2", "ln2_g", "ln2_b")
EMB_TENSORS = ("emb.word", "emb.pos", "emb.type", "emb.ln_g", "emb.ln_b")
HEAD_TENSORS = ("head.wt", "head.bt", "head.ln_g", "head.ln_b", "head.b_out")
NSP_TENSORS = ("pooler.w", "pooler.b", "nsp.w", "nsp.b")
IGNORE_LABEL = -100


class Ops:
    """Matrix-product hook: numpy matmul (host BLAS) or a literal triple loop."""

    def __init__(self, naive: bool = False):
        self.naive = naive

    def mm(self, a, b):
        if not self.naive:
            return a @ b
        m, k = a.shape
        k2, n = b.shape
        assert k == k2
        out = np.zeros((m, n), dtype=np.float64)
        for i in range(m):
            for j in range(n):
                s = 0.0
                for t in range(k):
                    s += float(a[i, t]) * float(b[t, j])
                out[i, j] = s
        return out


try:
    from scipy.special import erf as _erf   # library erf, exact to float64 rounding
except ImportError:  # pragma: no cover
    _erf = np.vectorize(math.erf, otypes=[np.float64])


def gelu(u):
    """erf form: u * Phi(u)."""
    return 0.5 * u * (1.0 + _erf(u / math.sqrt(2.0)))


def gelu_grad(u):
    """d/du [u Phi(u)] = Phi(u) + u phi(u)."""
    cdf = 0.5 * (1.0 + _erf(u / math.sqrt(2.0)))
    pdf = np.exp(-0.5 * u * u) / math.sqrt(2.0 * math.pi)
    return cdf + u * pdf


def layer_norm(z, g, b, eps):
    """Row-wise LayerNorm with biased variance. Returns y and (xhat, rstd) for the backward."""
    mu = z.mean(axis=-1, keepdims=True)
    var = ((z - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (z - mu) * rstd
    return xhat * g + b, (xhat, rstd)


def layer_norm_backward(dy, g, cache):
    xhat, rstd = cache
    dg = (dy * xhat).sum(axis=0)
    db = dy.sum(axis=0)
    dxh = dy * g
    dz = (dxh - dxh.mean(axis=-1, keepdims=True) - xhat * (dxh * xhat).mean(axis=-1, keepdims=True)) * rstd
    return dz, dg, db


def softmax_rows(a):
    m = a.max(axis=-1, keepdims=True)
    e = np.exp(a - m)
    return e / e.sum(axis=-1, keepdims=True)


def layers_per_group(cfg) -> int:
    return max(1, int(getattr(cfg, "layers_per_group", 1)))


def param_prefix(cfg, i: int) -> str:
    """Name prefix of the parameter set layer i uses: its own (BERT) or its group's (Section 3.3)."""
    return f"layer{i // layers_per_group(cfg)}."


def to_f64(params):
    return {k: np.asarray(v, dtype=np.float64) for k, v in params.items()}


# ----------------------------------------------------------------------------------------------
# dropout (BERT's dropout, adopted by reference in Section 4.1: probability 0.1 on the embedding
# output, the attention probabilities, the attention output and the feed-forward output)
# ----------------------------------------------------------------------------------------------
# The keep decisions come from a counter-based generator so that any implementation can reproduce
# them bit for bit: the SplitMix64 output function (Steele, Lea, Flood 2014) applied to
# key + quad * GOLDEN, where quad = element_index // 4 and the four 16-bit fields of the 64-bit
# result decide elements 4*quad .. 4*quad+3 (field j = bits 16j..16j+15): keep iff field >= thr,
# thr = round(p * 65536).  Kept values are scaled by 1 / (1 - p).  The key mixes the user's seed
# with (step, layer, site); element_index is the C-order index in the tensor the mask applies to.
GOLDEN = 0x9E3779B97F4A7C15
_M64 = (1 << 64) - 1
SITE_EMBEDDING, SITE_ATTN_PROBS, SITE_ATTN_OUT, SITE_FFN_OUT = 0, 1, 2, 3


def mix64(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def mix64_array(z):
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def dropout_key(seed: int, step: int, layer: int, site: int) -> int:
    stream = (step << 20) | (layer << 4) | site
    return mix64(seed ^ mix64(stream + GOLDEN))


class Dropout:
    """Dropout settings of one step: probability, seed and step number."""

    def __init__(self, p: float, seed: int, step: int):
        self.p, self.seed, self.step = float(p), int(seed), int(step)
        self.thr = int(round(self.p * 65536.0))
        self.scale = 1.0 / (1.0 - self.p)

    def mask(self, layer: int, site: int, shape):
        """Array of `shape` holding 0 (dropped) or 1/(1-p) (kept)."""
        n = int(np.prod(shape))
        key = dropout_key(self.seed, self.step, layer, site)
        quads = np.arange((n + 3) // 4, dtype=np.uint64)
        with np.errstate(over="ignore"):
            r = mix64_array(np.uint64(key) + quads * np.uint64(GOLDEN))
        fields = np.stack([(r >> np.uint64(16 * j)) & np.uint64(0xFFFF) for j in range(4)], axis=1).reshape(-1)[:n]
        return np.where(fields >= np.uint64(self.thr), self.scale, 0.0).reshape(shape)


# ----------------------------------------------------------------------------------------------
# forward
# ----------------------------------------------------------------------------------------------
def embed_forward(cfg, P, batch, drop=None):
    ids = np.asarray(batch["input_ids"]).reshape(-1)
    tt = np.asarray(batch["token_type_ids"]).reshape(-1)
    B, S = np.asarray(batch["input_ids"]).shape
    pos = np.tile(np.arange(S), B)
    z = P["emb.word"][ids] + P["emb.pos"][pos] + P["emb.type"][tt]
    x0, ln = layer_norm(z, P["emb.ln_g"], P["emb.ln_b"], cfg.ln_eps)
    mE = None
    if drop is not None:
        mE = drop.mask(0, SITE_EMBEDDING, x0.shape)
        x0 = x0 * mE
    return x0, {"ids": ids, "tt": tt, "pos": pos, "ln": ln, "mE": mE}


def layer_forward(cfg, P, i, X, key_bias, B, S, ops, drop=None):
    """One post-LN encoder layer. X is [T, H]; key_bias is [B, S] (0 for tokens, mask_bias for padding).

    In the grouped variant of Section 3.3 layer i uses the parameter set of its group, layer{i // g}.*."""
    p = param_prefix(cfg, i)
    H, nh = cfg.hidden, cfg.n_heads
    dh = H // nh
    Q = ops.mm(X, P[p + "wq"].T) + P[p + "bq"]
    K = ops.mm(X, P[p + "wk"].T) + P[p + "bk"]
    V = ops.mm(X, P[p + "wv"].T) + P[p + "bv"]
    C = np.empty_like(X)
    Pr = np.empty((B, nh, S, S), dtype=np.float64)
    scale = 1.0 / math.sqrt(dh)
    mA = drop.mask(i, SITE_ATTN_PROBS, (B, nh, S, S)) if drop is not None else None
    mO = drop.mask(i, SITE_ATTN_OUT, X.shape) if drop is not None else None
    mF = drop.mask(i, SITE_FFN_OUT, X.shape) if drop is not None else None
    for b in range(B):
        rows = slice(b * S, (b + 1) * S)
        for h in range(nh):
            cols = slice(h * dh, (h + 1) * dh)
            A = ops.mm(Q[rows, cols], K[rows, cols].T) * scale + key_bias[b][None, :]
            Pbh = softmax_rows(A)
            Pr[b, h] = Pbh
            Pd = Pbh if mA is None else Pbh * mA[b, h]
            C[rows, cols] = ops.mm(Pd, V[rows, cols])
    O = ops.mm(C, P[p + "wo"].T) + P[p + "bo"]
    if mO is not None:
        O = O * mO
    X1, ln1 = layer_norm(X + O, P[p + "ln1_g"], P[p + "ln1_b"], cfg.ln_eps)
    U = ops.mm(X1, P[p + "w1"].T) + P[p + "b1"]
    G = gelu(U)
    D = ops.mm(G, P[p + "w2"].T) + P[p + "b2"]
    if mF is not None:
        D = D * mF
    X2, ln2 = layer_norm(X1 + D, P[p + "ln2_g"], P[p + "ln2_b"], cfg.ln_eps)
    cache = {"X": X, "Q": Q, "K": K, "V": V, "P": Pr, "C": C, "ln1": ln1, "X1": X1, "U": U, "G": G, "ln2": ln2,
             "mA": mA, "mO": mO, "mF": mF}
    return X2, cache


def masked_rows(batch):
    """Ascending flat positions with a label, and the labels there (integer, unique)."""
    lab = np.asarray(batch["labels"]).reshape(-1)
    pos = np.flatnonzero(lab != IGNORE_LABEL)
    return pos.astype(np.int64), lab[pos].astype(np.int64)


def projection_matrix(P):
    """The word matrix as the output projection sees it.  It is the tied matrix `emb.word` itself unless the
    caller supplies `head.proj_word`: a diagnostic input for comparisons with a reduced-precision
    implementation whose projection reads a rounded copy of the matrix while its embedding lookup reads the
    unrounded one (the gradient still goes to the one tied matrix)."""
    return P.get("head.proj_word", P["emb.word"])


def head_forward(cfg, P, XL, pos, Y, ops):
    Xm = XL[pos]
    Ut = ops.mm(Xm, P["head.wt"].T) + P["head.bt"]
    Gt = gelu(Ut)
    Hm, ln = layer_norm(Gt, P["head.ln_g"], P["head.ln_b"], cfg.ln_eps)
    Z = ops.mm(Hm, projection_matrix(P).T) + P["head.b_out"]
    zmax = Z.max(axis=-1, keepdims=True)
    lse = (zmax + np.log(np.exp(Z - zmax).sum(axis=-1, keepdims=True)))[:, 0]
    M = len(pos)
    losses = lse - Z[np.arange(M), Y]
    loss = losses.sum() / M
    return loss, {"Xm": Xm, "Ut": Ut, "Gt": Gt, "Hm": Hm, "ln": ln, "Z": Z, "lse": lse, "pos": pos, "Y": Y}


def nsp_forward(cfg, P, XL, B, S, Ynsp, ops):
    """Next-sentence head (Section 4.1 keeps BERT's second objective): pooler = tanh(dense) of every
    sequence's first token, a two-way classifier on it, mean cross-entropy over the batch."""
    cls = np.arange(B) * S
    Xc = XL[cls]
    Pl = np.tanh(ops.mm(Xc, P["pooler.w"].T) + P["pooler.b"])
    Z = ops.mm(Pl, P["nsp.w"].T) + P["nsp.b"]
    zmax = Z.max(axis=-1, keepdims=True)
    lse = (zmax + np.log(np.exp(Z - zmax).sum(axis=-1, keepdims=True)))[:, 0]
    loss = (lse - Z[np.arange(B), Ynsp]).sum() / B
    return loss, {"cls": cls, "Xc": Xc, "Pl": Pl, "Z": Z, "lse": lse, "Y": Ynsp}


def nsp_backward(cfg, P, nc, ops):
    B = len(nc["cls"])
    dZ = np.exp(nc["Z"] - nc["lse"][:, None])
    dZ[np.arange(B), nc["Y"]] -= 1.0
    dZ /= B
    g = {"nsp.w": ops.mm(dZ.T, nc["Pl"]), "nsp.b": dZ.sum(axis=0)}
    dU = ops.mm(dZ, P["nsp.w"]) * (1.0 - nc["Pl"] ** 2)
    g["pooler.w"] = ops.mm(dU.T, nc["Xc"])
    g["pooler.b"] = dU.sum(axis=0)
    return ops.mm(dU, P["pooler.w"]), g          # gradient of the first-token rows of the last layer's output


def forward(cfg, params, batch, n_layers=None, ops=None, keep_from=0, prefix_at=None, drop=None):
    """Forward through the embedding block, layers 0..n_layers-1 and the masked-LM head.

    Layer caches below `keep_from` are dropped (those layers run forward only).
    `prefix_out` in the returned cache is the input of layer `prefix_at` (default keep_from),
    i.e. the output of the frozen prefix.
    """
    ops = ops or Ops()
    P = to_f64(params)
    n_layers = cfg.n_layers if n_layers is None else n_layers
    prefix_at = keep_from if prefix_at is None else prefix_at
    ids = np.asarray(batch["input_ids"])
    B, S = ids.shape
    key_bias = (1.0 - np.asarray(batch["attn_mask"], dtype=np.float64)) * cfg.mask_bias
    X, emb_cache = embed_forward(cfg, P, batch, drop)
    layer_caches = [None] * n_layers
    prefix_out = None
    for i in range(n_layers):
        if i == prefix_at:
            prefix_out = X
        X, c = layer_forward(cfg, P, i, X, key_bias, B, S, ops, drop)
        if i >= keep_from:
            layer_caches[i] = c
    pos, Y = masked_rows(batch)
    if len(pos) == 0:
        raise ValueError("batch has no predicted position")
    loss, head_cache = head_forward(cfg, P, X, pos, Y, ops)
    nsp_cache = None
    if getattr(cfg, "nsp", False):              # the two objectives are added
        nsp_loss, nsp_cache = nsp_forward(cfg, P, X, B, S, np.asarray(batch["nsp_labels"], dtype=np.int64), ops)
        loss = loss + nsp_loss
    cache = {"P64": P, "B": B, "S": S, "T": B * S, "n_layers": n_layers, "emb": emb_cache, "layers": layer_caches,
             "head": head_cache, "nsp": nsp_cache, "XL": X, "prefix_out": prefix_out, "keep_from": keep_from}
    return loss, cache


# ----------------------------------------------------------------------------------------------
# backward
# ----------------------------------------------------------------------------------------------
def head_backward(cfg, P, hc, T, ops):
    M = len(hc["pos"])
    Z = hc["Z"]
    dZ = np.exp(Z - hc["lse"][:, None])
    dZ[np.arange(M), hc["Y"]] -= 1.0
    dZ /= M
    g = {}
    g["head.b_out"] = dZ.sum(axis=0)
    g_word_head = ops.mm(dZ.T, hc["Hm"])          # contribution to the tied word matrix
    dHm = ops.mm(dZ, projection_matrix(P))
    dGt, g["head.ln_g"], g["head.ln_b"] = layer_norm_backward(dHm, P["head.ln_g"], hc["ln"])
    dUt = dGt * gelu_grad(hc["Ut"])
    g["head.wt"] = ops.mm(dUt.T, hc["Xm"])
    g["head.bt"] = dUt.sum(axis=0)
    dXm = ops.mm(dUt, P["head.wt"])
    dXL = np.zeros((T, cfg.hidden), dtype=np.float64)
    dXL[hc["pos"]] = dXm
    return dXL, g, g_word_head, dZ


def layer_backward(cfg, P, i, c, dX2, B, S, ops):
    p = param_prefix(cfg, i)
    H, nh = cfg.hidden, cfg.n_heads
    dh = H // nh
    scale = 1.0 / math.sqrt(dh)
    g = {}
    dZ2, g[p + "ln2_g"], g[p + "ln2_b"] = layer_norm_backward(dX2, P[p + "ln2_g"], c["ln2"])
    dD = dZ2 if c.get("mF") is None else dZ2 * c["mF"]
    g[p + "w2"] = ops.mm(dD.T, c["G"])
    g[p + "b2"] = dD.sum(axis=0)
    dG = ops.mm(dD, P[p + "w2"])
    dU = dG * gelu_grad(c["U"])
    g[p + "w1"] = ops.mm(dU.T, c["X1"])
    g[p + "b1"] = dU.sum(axis=0)
    dX1 = ops.mm(dU, P[p + "w1"]) + dZ2
    dZ1, g[p + "ln1_g"], g[p + "ln1_b"] = layer_norm_backward(dX1, P[p + "ln1_g"], c["ln1"])
    dO = dZ1 if c.get("mO") is None else dZ1 * c["mO"]
    g[p + "wo"] = ops.mm(dO.T, c["C"])
    g[p + "bo"] = dO.sum(axis=0)
    dC = ops.mm(dO, P[p + "wo"])
    dQ = np.empty_like(dC)
    dK = np.empty_like(dC)
    dV = np.empty_like(dC)
    for b in range(B):
        rows = slice(b * S, (b + 1) * S)
        for h in range(nh):
            cols = slice(h * dh, (h + 1) * dh)
            Pbh = c["P"][b, h]
            dCbh = dC[rows, cols]
            mA = None if c.get("mA") is None else c["mA"][b, h]
            Pd = Pbh if mA is None else Pbh * mA
            dV[rows, cols] = ops.mm(Pd.T, dCbh)
            dP = ops.mm(dCbh, c["V"][rows, cols].T)
            if mA is not None:
                dP = dP * mA
            dA = Pbh * (dP - (dP * Pbh).sum(axis=-1, keepdims=True))
            dQ[rows, cols] = ops.mm(dA, c["K"][rows, cols]) * scale
            dK[rows, cols] = ops.mm(dA.T, c["Q"][rows, cols]) * scale
    X = c["X"]
    for nm, dY in (("q", dQ), ("k", dK), ("v", dV)):
        g[p + "w" + nm] = ops.mm(dY.T, X)
        g[p + "b" + nm] = dY.sum(axis=0)
    dX = ops.mm(dQ, P[p + "wq"]) + ops.mm(dK, P[p + "wk"]) + ops.mm(dV, P[p + "wv"]) + dZ1
    return dX, g


def embed_backward(cfg, P, ec, dX0):
    g = {}
    if ec.get("mE") is not None:
        dX0 = dX0 * ec["mE"]
    dz, g["emb.ln_g"], g["emb.ln_b"] = layer_norm_backward(dX0, P["emb.ln_g"], ec["ln"])
    gw = np.zeros_like(P["emb.word"])
    gp = np.zeros_like(P["emb.pos"])
    gt = np.zeros_like(P["emb.type"])
    np.add.at(gw, ec["ids"], dz)
    np.add.at(gp, ec["pos"], dz)
    np.add.at(gt, ec["tt"], dz)
    g["emb.pos"], g["emb.type"] = gp, gt
    return g, gw


def backward(cfg, cache, ops=None, stop_layer=0, with_embeddings=True):
    """Reverse-mode gradients of the loss for layers >= stop_layer, the head and (optionally) the embeddings."""
    ops = ops or Ops()
    P = cache["P64"]
    B, S, T = cache["B"], cache["S"], cache["T"]
    dX, grads, g_word_head, _ = head_backward(cfg, P, cache["head"], T, ops)
    if cache.get("nsp") is not None:
        dXc, g = nsp_backward(cfg, P, cache["nsp"], ops)
        dX[cache["nsp"]["cls"]] += dXc
        grads.update(g)
    for i in range(cache["n_layers"] - 1, stop_layer - 1, -1):
        dX, g = layer_backward(cfg, P, i, cache["layers"][i], dX, B, S, ops)
        for name, val in g.items():      # layers of one group share their tensors: their gradients add up
            grads[name] = grads[name] + val if name in grads else val
    if with_embeddings:
        assert stop_layer == 0
        ge, gw_in = embed_backward(cfg, P, cache["emb"], dX)
        grads.update(ge)
        grads["emb.word"] = gw_in + g_word_head   # tied matrix: input gather + output projection
    return grads


def stage_tensor_names(frozen_layers, trainable_layers, train_embeddings, group=1):
    names = list(EMB_TENSORS) if train_embeddings else []
    for i in range(frozen_layers // group, (frozen_layers + trainable_layers) // group):
        names += [f"layer{i}.{t}" for t in LAYER_TENSORS]
    names += list(HEAD_TENSORS)
    return names


def stage_step(cfg, params, batch, frozen_layers, trainable_layers, train_embeddings=False, ops=None,
               full_backprop=False, drop=None):
    """Loss and gradients of one MSLT stage step (Section 3.2).

    Layers [0, frozen) run forward only; layers [frozen, frozen+trainable) and the
    output layer get gradients; the embedding block (with the tied word matrix) gets
    gradients only when `train_embeddings` (first stage, retraining).  With
    full_backprop the backward runs through every layer and the trainable slice is
    taken afterwards, which is the plain definition; without it the backward stops at
    the lowest trainable layer, which by the chain rule yields the same slice.
    `drop` (a Dropout, or None) switches dropout on in frozen and trainable layers alike.
    """
    if trainable_layers < 1 or frozen_layers < 0 or frozen_layers + trainable_layers > cfg.n_layers:
        raise ValueError("bad layer split")
    if train_embeddings and frozen_layers != 0:
        raise ValueError("embeddings train only when nothing is frozen")
    n = frozen_layers + trainable_layers
    keep_from = 0 if full_backprop else frozen_layers
    loss, cache = forward(cfg, params, batch, n_layers=n, ops=ops, keep_from=keep_from, prefix_at=frozen_layers,
                          drop=drop)
    if full_backprop:
        g_all = backward(cfg, cache, ops=ops, stop_layer=0, with_embeddings=True)
    else:
        g_all = backward(cfg, cache, ops=ops, stop_layer=frozen_layers, with_embeddings=train_embeddings)
    g = layers_per_group(cfg)
    if frozen_layers % g or trainable_layers % g:
        raise ValueError("frozen and trainable layers must be whole groups")
    names = stage_tensor_names(frozen_layers, trainable_layers, train_embeddings, g)
    if getattr(cfg, "nsp", False):
        names += list(NSP_TENSORS)
    grads = {k: g_all[k] for k in names}
    info = {"pos": cache["head"]["pos"], "labels": cache["head"]["Y"], "prefix_out": cache["prefix_out"],
            "XL": cache["XL"], "cache": cache}
    return loss, grads, info


# ----------------------------------------------------------------------------------------------
# optimizers (textbook Adam with decoupled weight decay; LAMB = same direction scaled per tensor)
# ----------------------------------------------------------------------------------------------
def decays(name: str) -> bool:
    """Weight decay applies to matrices and embedding tables, not to biases or LayerNorm parameters."""
    leaf = name.split(".")[-1]
    return leaf in ("word", "pos", "type", "wq", "wk", "wv", "wo", "w1", "w2", "wt", "w")


def new_opt_state(params):
    return {k: {"m": np.zeros_like(np.asarray(v, dtype=np.float64)),
                "v": np.zeros_like(np.asarray(v, dtype=np.float64)), "t": 0} for k, v in params.items()}


def optimizer_update(params, grads, state, kind="adam", lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-6,
                     weight_decay=0.01, bias_correction=True):
    """Update exactly the tensors in `grads`; every other tensor and its state stay untouched.

    m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g^2;  mhat, vhat bias-corrected with the
    tensor's own step count;  u = mhat / (sqrt(vhat) + eps) + wd * w.
    Adam: w -= lr u.   LAMB: w -= lr * (|w| / |u|) u, ratio 1 if either norm is 0.
    Returns new float64 params dict (inputs are not modified) and per-tensor trust ratios.
    """
    out = {k: np.array(v, dtype=np.float64, copy=True) for k, v in params.items()}
    ratios = {}
    for name, g in grads.items():
        st = state[name]
        g = np.asarray(g, dtype=np.float64)
        w = out[name]
        st["t"] += 1
        t = st["t"]
        st["m"] = beta1 * st["m"] + (1.0 - beta1) * g
        st["v"] = beta2 * st["v"] + (1.0 - beta2) * g * g
        if bias_correction:
            mhat = st["m"] / (1.0 - beta1 ** t)
            vhat = st["v"] / (1.0 - beta2 ** t)
        else:
            mhat, vhat = st["m"], st["v"]
        u = mhat / (np.sqrt(vhat) + eps)
        if decays(name) and weight_decay != 0.0:
            u = u + weight_decay * w
        r = 1.0
        if kind == "lamb":
            wn = math.sqrt(float((w * w).sum()))
            un = math.sqrt(float((u * u).sum()))
            r = wn / un if (wn > 0.0 and un > 0.0) else 1.0
        elif kind != "adam":
            raise ValueError(kind)
        ratios[name] = r
        out[name] = w - lr * r * u
    return out, ratios


def grow(params, n_present, n_new):
    """Stack growth (Section 3.2): new layer n_present+i is a copy of layer n_present-n_new+i.
    With grouped layers (Section 3.3) the counts are in parameter sets (groups)."""
    out = dict(params)
    for i in range(n_new):
        for t in LAYER_TENSORS:
            out[f"layer{n_present + i}.{t}"] = np.array(params[f"layer{n_present - n_new + i}.{t}"], copy=True)
    return out
