"""Shared helpers of the GPU parity tests: run one stage step through the C ABI and through the
oracle on the same seeded inputs and compare element by element."""
import numpy as np

from oracle import mslt_oracle as O
from paper_2011_13635_amd import binding, synth

# tolerances: loss and gradients relative 1e-4 in fp32 mode, relative 2e-2 (max-norm) in bf16 mode
TOL = {0: 1e-4, 1: 2e-2}


# second bf16-mode tolerance: against the oracle fed with the very bf16-rounded matrices the matrix cores consume,
# which leaves only the arithmetic of the kernels (rounded activations and gradients, summation order)
KERNEL_TOL = 1.2e-2


def bf16_round(a):
    """fp32 -> bf16 -> fp32, round to nearest even (numpy bit arithmetic)."""
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    u = a32.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a32.shape)


def rounded_weights(W):
    """The parameters as the library's bf16 mode reads them: the matrices that feed the matrix cores rounded to
    bf16 (encoder and head matrices, and the word matrix in its role as output projection), everything else
    (biases, LayerNorm parameters, the embedding tables of the lookup) as the fp32 masters."""
    out = dict(W)
    for n, v in W.items():
        if v.ndim == 2 and not n.startswith("emb."):
            out[n] = bf16_round(v)
    out["head.proj_word"] = bf16_round(W["emb.word"])
    return out


def make_model(shape, B, S, precision, max_predictions=0):
    cfg = binding.make_config(shape, B, S, precision, max_predictions)
    return binding.Model(cfg)


def grads_dict(model, shape, f, k, emb):
    flat = model.mslt_get_grads()
    return synth.unpack_weights(shape, flat, synth.trainable_names(shape, f, k, emb))


def rel_errors(g_gpu, g_ref):
    """Per-tensor max-norm relative error |g_gpu - g_ref|_inf / |g_ref|_inf.

    The key bias has a mathematically zero gradient (softmax is invariant to a per-row shift of
    the scores), so its error is measured against the query-bias gradient of the same layer.
    """
    out = {}
    for name, ref in g_ref.items():
        ref = np.asarray(ref, dtype=np.float64)
        got = np.asarray(g_gpu[name], dtype=np.float64)
        assert got.shape == ref.shape, name
        scale = np.abs(ref).max()
        if name.endswith(".bk"):
            scale = max(scale, np.abs(g_ref[name[:-2] + "bq"]).max())
        out[name] = np.abs(got - ref).max() / max(scale, 1e-30)
    return out


def run_case(shape, B, S, f, k, emb, precision, ragged=False, seed=0, std=0.02, perturb=0.0, full_backprop=True,
             model=None, weights=None, dropout=None, rounded_oracle=False):
    """Returns dict with loss / grads of both sides for one step on seeded inputs."""
    W = weights if weights is not None else synth.make_weights(shape, seed=seed, std=std, perturb=perturb)
    batch = synth.make_batch(shape, B, S, seed=seed + 1, ragged=ragged)
    own = model is None
    if own:
        model = make_model(shape, B, S, precision)
    model.mslt_load_params(synth.pack_weights(shape, W))
    cb = model.device_batch(batch)
    drop = None
    if dropout is not None:            # (p, seed, step): both sides derive the same keep decisions from it
        model.mslt_set_dropout(*dropout)
        drop = O.Dropout(*dropout)
    loss = model.mslt_stage_step(f, k, emb, cb)
    g = grads_dict(model, shape, f, k, emb)
    pos, lab = model.mslt_debug_masked()
    prefix = model.mslt_debug_prefix_output(B, S)
    ref_loss, ref_g, info = O.stage_step(shape, W, batch, f, k, emb, full_backprop=full_backprop, drop=drop)
    out = {"model": model, "W": W, "batch": batch, "cb": cb, "loss": loss, "grads": g, "pos": pos, "lab": lab,
           "prefix": prefix, "ref_loss": ref_loss, "ref_grads": ref_g, "ref_info": info}
    if rounded_oracle:     # the same step of the oracle on the matrices as bf16 mode reads them
        out["rnd_loss"], out["rnd_grads"], _ = O.stage_step(shape, rounded_weights(W), batch, f, k, emb,
                                                            full_backprop=full_backprop, drop=drop)
    return out


def assert_parity(r, precision, label="", grad_tol=None):
    """grad_tol: bound on the gradients against the oracle on the fp32 masters when it is not TOL[precision]
    (a case that also carries the oracle on the rounded matrices, where the quantisation of the matrices alone
    takes most of 2e-2; the bound against the rounded matrices is then the sharp one)."""
    tol = TOL[precision]
    gtol = tol if grad_tol is None else grad_tol
    assert grad_tol is None or "rnd_grads" in r, "a wider bound against the masters needs the rounded-matrices oracle"
    # integer work: bit-exact
    assert np.array_equal(r["pos"], r["ref_info"]["pos"].astype(np.int32)), label
    assert np.array_equal(r["lab"], r["ref_info"]["labels"].astype(np.int32)), label
    assert np.array_equal(r["pos"], r["batch"]["masked_positions"]), label
    lerr = abs(r["loss"] - r["ref_loss"]) / abs(r["ref_loss"])
    assert lerr < tol, (label, "loss", r["loss"], r["ref_loss"], lerr)
    errs = rel_errors(r["grads"], r["ref_grads"])
    worst = max(errs, key=errs.get)
    assert errs[worst] < gtol, (label, worst, errs[worst], sorted(errs.items(), key=lambda kv: -kv[1])[:5])
    assert set(r["grads"]) == set(r["ref_grads"])
    # frozen-prefix output
    ref_p = r["ref_info"]["prefix_out"]
    perr = np.abs(r["prefix"] - ref_p).max() / np.abs(ref_p).max()
    assert perr < tol, (label, "prefix", perr)
    if "rnd_grads" in r:
        kerrs = rel_errors(r["grads"], r["rnd_grads"])
        kworst = max(kerrs, key=kerrs.get)
        assert kerrs[kworst] < KERNEL_TOL, (label, "against the oracle on rounded matrices", kworst, kerrs[kworst])
        assert abs(r["loss"] - r["rnd_loss"]) / abs(r["rnd_loss"]) < KERNEL_TOL, (label, "loss, rounded matrices")
        return lerr, errs[worst], worst, kerrs[kworst], kworst
    return lerr, errs[worst], worst
