"""Thin ctypes binding of the learning-to-hash trainer in ``libhata.so`` (C ABI declared in
``include/hata_train.h``).

Argument marshalling only: the loss, its gradient, the optimiser and the construction of the
training labels run in the HIP kernels.  torch allocates device memory and supplies the stream.
No CPU fallback.
"""
from __future__ import annotations

import ctypes

from . import hata as _hata

EXPORTS = ("hata_train_workspace_bytes", "hata_train_create", "hata_train_destroy", "hata_train_step",
           "hata_train_make_labels")
BLOCK = 128  # HATA_TRAIN_BLOCK: triplets per block of the per-query balance term


class hata_train_config(ctypes.Structure):
    _fields_ = [("d", ctypes.c_int32), ("r", ctypes.c_int32), ("n_max", ctypes.c_int32)]


class hata_train_hparams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_float) for n in ("sigma", "eps", "eta", "lam", "scale_sim", "scale_bal",
                                               "lr", "momentum", "weight_decay")]


def default_hparams(n: int, mean_forms: bool = True) -> hata_train_hparams:
    """Hyper-parameter table of App. B.2; mean_forms scales the two data terms by 1/n and 1/n^2."""
    return hata_train_hparams(0.1, 0.01, 2.0, 1.0, 1.0 / n if mean_forms else 1.0,
                              1.0 / (n * n) if mean_forms else 1.0, 0.1, 0.9, 1e-6)


_bound = False


def _lib():
    global _bound
    lib = _hata.load_library()
    if not _bound:
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        lib.hata_train_workspace_bytes.argtypes = [ctypes.POINTER(hata_train_config), ctypes.POINTER(ctypes.c_size_t)]
        lib.hata_train_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(hata_train_config), vp, ctypes.c_size_t]
        lib.hata_train_destroy.argtypes = [vp]
        lib.hata_train_step.argtypes = [vp, vp, vp, vp, i32, vp, i32, vp, vp, ctypes.POINTER(hata_train_hparams),
                                        vp, vp, vp]
        lib.hata_train_make_labels.argtypes = [vp, vp, vp, i32, vp, vp]
        for n in EXPORTS:
            getattr(lib, n).restype = ctypes.c_int
        _bound = True
    return lib


class TrainContext:
    """Owns a hata_train_ctx and the torch-allocated workspace it points into."""

    def __init__(self, d: int, r: int, n_max: int, device="cuda:0"):
        import torch
        lib = _lib()
        if not torch.cuda.is_available():
            raise _hata.HataError("no GPU visible: the trainer has no CPU fallback")
        self.cfg = hata_train_config(d, r, n_max)
        nbytes = ctypes.c_size_t(0)
        _hata._check(lib.hata_train_workspace_bytes(ctypes.byref(self.cfg), ctypes.byref(nbytes)),
                     "hata_train_workspace_bytes")
        self.workspace = torch.empty(nbytes.value + 256, dtype=torch.uint8, device=device)
        ws = (self.workspace.data_ptr() + 255) // 256 * 256
        self._h = ctypes.c_void_p(None)
        _hata._check(lib.hata_train_create(ctypes.byref(self._h), ctypes.byref(self.cfg),
                                           ctypes.c_void_p(ws), nbytes.value), "hata_train_create")
        self.workspace_bytes = nbytes.value

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            _lib().hata_train_destroy(self._h)
            self._h = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def hata_train_step(self, Q, K, s, n, W, v, hp: hata_train_hparams, grad=None, loss=None, stream=None,
                        block_query=None, n_queries=1):
        _hata._check(_lib().hata_train_step(self._h, _hata._ptr(Q), _hata._ptr(K), _hata._ptr(s), n,
                                            _hata._ptr(block_query), n_queries, _hata._ptr(W), _hata._ptr(v),
                                            ctypes.byref(hp), _hata._ptr(grad), _hata._ptr(loss),
                                            _hata._stream(stream)), "hata_train_step")

    def hata_train_make_labels(self, q, K, m, s, stream=None):
        _hata._check(_lib().hata_train_make_labels(self._h, _hata._ptr(q), _hata._ptr(K), m, _hata._ptr(s),
                                                   _hata._stream(stream)), "hata_train_make_labels")
