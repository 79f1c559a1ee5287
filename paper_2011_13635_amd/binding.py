"""ctypes binding of libmslt.so: same names as include/mslt.h, argument marshalling only.

PyTorch is used for device memory (the four arenas, the batch tensors) and the stream.
Every step of the path runs inside the library's HIP kernels; there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmslt.so")

EXPORTS = [
    "mslt_query_sizes", "mslt_init_model", "mslt_tensor_table", "mslt_load_params", "mslt_get_params",
    "mslt_stage_step", "mslt_grad_count", "mslt_get_grads", "mslt_apply_update", "mslt_apply_update_static",
    "mslt_train_step",
    "mslt_set_dropout", "mslt_debug_masked",
    "mslt_debug_prefix_output", "mslt_grow", "mslt_sync", "mslt_destroy", "mslt_last_error",
    "mslt_profile_enable", "mslt_profile_read", "mslt_debug_gemm",
]

MSLT_OK, MSLT_ERR_ARG, MSLT_ERR_STATE, MSLT_ERR_DATA, MSLT_ERR_HIP, MSLT_ERR_NONFINITE = 0, -1, -2, -3, -4, -5


class MsltError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"mslt error {code}: {msg}")
        self.code = code


class Config(C.Structure):
    _fields_ = [("n_layers_max", C.c_int), ("hidden", C.c_int), ("n_heads", C.c_int), ("ffn", C.c_int),
                ("vocab", C.c_int), ("max_pos", C.c_int), ("type_vocab", C.c_int), ("max_batch", C.c_int),
                ("max_seq", C.c_int), ("max_predictions", C.c_int), ("precision", C.c_int),
                ("ln_eps", C.c_float), ("mask_bias", C.c_float), ("layers_per_group", C.c_int),
                ("with_nsp", C.c_int), ("max_trainable_layers", C.c_int)]


class Batch(C.Structure):
    _fields_ = [("input_ids", C.c_void_p), ("token_type_ids", C.c_void_p), ("attn_mask", C.c_void_p),
                ("labels", C.c_void_p), ("batch", C.c_int), ("seq", C.c_int), ("nsp_labels", C.c_void_p)]


class Opt(C.Structure):
    _fields_ = [("kind", C.c_int), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("weight_decay", C.c_float), ("bias_correction", C.c_int)]


class TensorDesc(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("layer", C.c_int), ("rows", C.c_int), ("cols", C.c_int),
                ("decays", C.c_int), ("offset", C.c_size_t), ("count", C.c_size_t)]


class ProfileEntry(C.Structure):
    _fields_ = [("name", C.c_char * 24), ("launches", C.c_int), ("ms", C.c_double), ("flops", C.c_double),
                ("bytes", C.c_double)]


_lib = None


def load_library():
    """Loads the in-tree shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2011_13635_amd.build)")
    lib = C.CDLL(LIB_PATH)
    vp, sz = C.c_void_p, C.c_size_t
    P = C.POINTER
    lib.mslt_query_sizes.argtypes = [P(Config), P(sz), P(sz), P(sz), P(sz)]
    lib.mslt_init_model.argtypes = [P(Config), vp, vp, vp, vp, vp, P(vp)]
    lib.mslt_tensor_table.argtypes = [vp, P(C.c_int), P(P(TensorDesc))]
    lib.mslt_load_params.argtypes = [vp, vp, sz]
    lib.mslt_get_params.argtypes = [vp, vp, sz]
    lib.mslt_stage_step.argtypes = [vp, C.c_int, C.c_int, C.c_int, P(Batch), P(C.c_float)]
    lib.mslt_grad_count.argtypes = [vp, P(sz)]
    lib.mslt_get_grads.argtypes = [vp, vp, sz]
    lib.mslt_apply_update.argtypes = [vp, P(Opt)]
    lib.mslt_apply_update_static.argtypes = [vp, P(Opt)]
    lib.mslt_train_step.argtypes = [vp, C.c_int, C.c_int, C.c_int, P(Batch), P(Opt), P(C.c_float)]
    lib.mslt_set_dropout.argtypes = [vp, C.c_float, C.c_uint64, C.c_uint64]
    lib.mslt_debug_masked.argtypes = [vp, vp, vp, P(C.c_int)]
    lib.mslt_debug_prefix_output.argtypes = [vp, vp, sz]
    lib.mslt_grow.argtypes = [vp, C.c_int, C.c_int]
    lib.mslt_profile_enable.argtypes = [vp, C.c_int]
    lib.mslt_profile_read.argtypes = [vp, P(ProfileEntry), C.c_int, P(C.c_int)]
    lib.mslt_sync.argtypes = [vp]
    lib.mslt_debug_gemm.argtypes = [vp, vp, vp, vp] + [C.c_int] * 11 + [vp, sz]
    lib.mslt_destroy.argtypes = [vp]
    lib.mslt_last_error.argtypes = []
    lib.mslt_last_error.restype = C.c_char_p
    for name in EXPORTS:
        if name != "mslt_last_error":
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _check(rc, allow=()):
    if rc != 0 and rc not in allow:
        raise MsltError(rc, load_library().mslt_last_error().decode())
    return rc


def make_config(shape, max_batch, max_seq, precision, max_predictions=0, max_trainable_layers=0) -> Config:
    """Config from a synth.ModelShape-like object (n_layers, hidden, n_heads, ffn, vocab, ...)."""
    return Config(shape.n_layers, shape.hidden, shape.n_heads, shape.ffn, shape.vocab, shape.max_pos,
                  shape.type_vocab, max_batch, max_seq, max_predictions, precision, shape.ln_eps, shape.mask_bias,
                  getattr(shape, "layers_per_group", 1), int(getattr(shape, "nsp", False)), max_trainable_layers)


def mslt_query_sizes(cfg: Config):
    a, b, c, d = C.c_size_t(), C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(load_library().mslt_query_sizes(C.byref(cfg), C.byref(a), C.byref(b), C.byref(c), C.byref(d)))
    return a.value, b.value, c.value, d.value


def adam(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-6, weight_decay=0.01, bias_correction=True) -> Opt:
    return Opt(0, lr, beta1, beta2, eps, weight_decay, int(bias_correction))


def lamb(lr=0.00088, beta1=0.9, beta2=0.999, eps=1e-6, weight_decay=0.01, bias_correction=True) -> Opt:
    return Opt(1, lr, beta1, beta2, eps, weight_decay, int(bias_correction))


def mslt_debug_gemm(a, b, c, M, N, K, a_kcontig, b_kcontig, kernel, tile_m=0, tile_n=0, tile_k=64, splitk=1,
                    partials=None, stream=None):
    """One product through a chosen kernel.  a, b: torch bf16 device tensors; c: bf16 or fp32 device tensor
    [M, N]; partials: uint8/fp32 device tensor for split-k.  Enqueues only."""
    import torch
    out_f32 = int(c.dtype == torch.float32)
    st = stream if stream is not None else torch.cuda.current_stream(a.device)
    pb = partials.numel() * partials.element_size() if partials is not None else 0
    _check(load_library().mslt_debug_gemm(C.c_void_p(st.cuda_stream), C.c_void_p(a.data_ptr()), C.c_void_p(b.data_ptr()),
                                          C.c_void_p(c.data_ptr()), M, N, K, int(a_kcontig), int(b_kcontig), out_f32, kernel,
                                          tile_m, tile_n, tile_k, splitk,
                                          C.c_void_p(partials.data_ptr()) if partials is not None else None, pb))


class Model:
    """Owns the torch device arenas and the opaque model handle.  Methods mirror the C calls."""

    def __init__(self, cfg: Config, device="cuda:0", stream=None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the MSLT library has no CPU path")
        self.lib = load_library()
        self.torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        sizes = mslt_query_sizes(cfg)
        self.sizes = sizes
        with torch.cuda.device(self.device):
            self.arenas = [torch.empty(max(s, 256), dtype=torch.uint8, device=self.device) for s in sizes]
            self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        h = C.c_void_p()
        _check(self.lib.mslt_init_model(C.byref(cfg), *[C.c_void_p(a.data_ptr()) for a in self.arenas],
                                        C.c_void_p(self.stream.cuda_stream), C.byref(h)))
        self.handle = h
        self._batch_keep = None
        n = C.c_int()
        tab = C.POINTER(TensorDesc)()
        _check(self.lib.mslt_tensor_table(self.handle, C.byref(n), C.byref(tab)))
        self.table = [(tab[i].name.decode(), tab[i].layer, tab[i].rows, tab[i].cols, tab[i].decays, tab[i].offset,
                       tab[i].count) for i in range(n.value)]
        self.packed_count = sum(t[6] for t in self.table)

    # -- parameters
    def mslt_load_params(self, flat: np.ndarray):
        flat = np.ascontiguousarray(flat, dtype=np.float32)
        _check(self.lib.mslt_load_params(self.handle, flat.ctypes.data_as(C.c_void_p), flat.size))

    def mslt_get_params(self) -> np.ndarray:
        out = np.empty(self.packed_count, dtype=np.float32)
        _check(self.lib.mslt_get_params(self.handle, out.ctypes.data_as(C.c_void_p), out.size))
        return out

    # -- batches
    def device_batch(self, batch) -> Batch:
        """Copies a host batch (dict of int arrays [B,S]) to the device; returns the C struct."""
        torch = self.torch
        B, S = batch["input_ids"].shape
        keep = [torch.as_tensor(np.ascontiguousarray(batch[k], dtype=np.int32)).to(self.device)
                for k in ("input_ids", "token_type_ids", "attn_mask", "labels")]
        nsp = None
        if "nsp_labels" in batch:
            nsp = torch.as_tensor(np.ascontiguousarray(batch["nsp_labels"], dtype=np.int32)).to(self.device)
        torch.cuda.synchronize(self.device)
        cb = Batch(*[C.c_void_p(t.data_ptr()) for t in keep], B, S, C.c_void_p(nsp.data_ptr()) if nsp is not None else None)
        keep.append(nsp)
        cb._keep = keep   # keep the tensors alive as long as the struct
        return cb

    # -- the step
    def mslt_stage_step(self, frozen_layers, trainable_layers, train_embeddings, cbatch: Batch, allow=()):
        loss = C.c_float()
        rc = _check(self.lib.mslt_stage_step(self.handle, frozen_layers, trainable_layers, int(train_embeddings),
                                             C.byref(cbatch), C.byref(loss)), allow)
        return loss.value if rc == 0 else rc

    def mslt_grad_count(self) -> int:
        n = C.c_size_t()
        _check(self.lib.mslt_grad_count(self.handle, C.byref(n)))
        return n.value

    def mslt_get_grads(self) -> np.ndarray:
        out = np.empty(self.mslt_grad_count(), dtype=np.float32)
        _check(self.lib.mslt_get_grads(self.handle, out.ctypes.data_as(C.c_void_p), out.size))
        return out

    def mslt_apply_update(self, opt: Opt):
        _check(self.lib.mslt_apply_update(self.handle, C.byref(opt)))

    def mslt_apply_update_static(self, opt: Opt):
        _check(self.lib.mslt_apply_update_static(self.handle, C.byref(opt)))

    def mslt_train_step(self, frozen_layers, trainable_layers, train_embeddings, cbatch: Batch, opt: Opt, allow=()):
        loss = C.c_float()
        rc = _check(self.lib.mslt_train_step(self.handle, frozen_layers, trainable_layers, int(train_embeddings),
                                             C.byref(cbatch), C.byref(opt), C.byref(loss)), allow)
        return loss.value if rc == 0 else rc

    def mslt_set_dropout(self, p: float, seed: int, step: int):
        _check(self.lib.mslt_set_dropout(self.handle, p, seed, step))

    def mslt_debug_masked(self):
        cap = self.cfg.max_predictions or self.cfg.max_batch * self.cfg.max_seq
        pos = np.empty(cap, dtype=np.int32)
        lab = np.empty(cap, dtype=np.int32)
        m = C.c_int()
        _check(self.lib.mslt_debug_masked(self.handle, pos.ctypes.data_as(C.c_void_p), lab.ctypes.data_as(C.c_void_p),
                                          C.byref(m)))
        return pos[:m.value].copy(), lab[:m.value].copy()

    def mslt_debug_prefix_output(self, batch, seq) -> np.ndarray:
        out = np.empty(batch * seq * self.cfg.hidden, dtype=np.float32)
        _check(self.lib.mslt_debug_prefix_output(self.handle, out.ctypes.data_as(C.c_void_p), out.size))
        return out.reshape(batch * seq, self.cfg.hidden)

    def mslt_grow(self, n_present, n_new):
        _check(self.lib.mslt_grow(self.handle, n_present, n_new))

    def mslt_profile_enable(self, on: bool):
        _check(self.lib.mslt_profile_enable(self.handle, int(on)))

    def mslt_profile_read(self):
        """Per kernel class since the last read: {name: dict(launches, ms, flops, bytes)} (classes that ran)."""
        buf = (ProfileEntry * 16)()
        n = C.c_int()
        _check(self.lib.mslt_profile_read(self.handle, buf, 16, C.byref(n)))
        return {buf[i].name.decode(): {"launches": buf[i].launches, "ms": buf[i].ms, "flops": buf[i].flops,
                                       "bytes": buf[i].bytes} for i in range(n.value) if buf[i].launches}

    def mslt_sync(self):
        _check(self.lib.mslt_sync(self.handle))

    def close(self):
        if self.handle:
            self.lib.mslt_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
