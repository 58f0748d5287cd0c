"""Thin ctypes binding of ``libhata.so`` (the C ABI declared in ``include/hata.h``).

Argument marshalling only: every step of the path runs in the HIP kernels behind the
C ABI.  torch is used for device memory and the stream handle, nothing else.  There is
no CPU fallback: if the library is missing or a call fails, an exception is raised.
Function names match the C entry points.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhata.so")

EXPORTS = (
    "hata_strerror", "hata_workspace_bytes", "hata_workspace_bytes_tuned", "hata_create", "hata_create_tuned",
    "hata_destroy", "hata_encode_keys", "hata_prepare_weights",
    "hata_prefill_write", "hata_prefill_write_paged", "hata_encode_query", "hata_hamming_score", "hata_topk", "hata_sparse_decode",
    "hata_sparse_decode_static", "hata_gather_rows", "hata_dense_decode", "hata_decode_step", "hata_select_step", "hata_decode_step_paged", "hata_step_plan", "hata_step_sub_batches", "hata_set_step_mode", "hata_keep_step_scores", "hata_set_wait_limit",
    "hata_check",
    "hata_host_device_pointer", "hata_step_buffers", "hata_probe_mfma_stream",
)


class HataError(RuntimeError):
    pass


class hata_config(ctypes.Structure):
    _fields_ = [
        ("B_max", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
        ("d", ctypes.c_int32), ("r", ctypes.c_int32), ("L_cap", ctypes.c_int32),
        ("k_max", ctypes.c_int32),
        ("kv_stride_b", ctypes.c_int64), ("kv_stride_h", ctypes.c_int64),
        ("kv_stride_n", ctypes.c_int64),
    ]


class hata_tuning(ctypes.Structure):
    _fields_ = [("chunk", ctypes.c_int32), ("attn_rows", ctypes.c_int32), ("par_merge", ctypes.c_int32),
                ("shared_device", ctypes.c_int32)]


_lib = None
_vp = ctypes.c_void_p
_i32 = ctypes.c_int32


def load_library(build_if_missing: bool = True) -> ctypes.CDLL:
    """Load libhata.so (building it with hipcc first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    # torch ships its own HIP runtime with the same soname as the system one; importing torch
    # first makes libhata.so bind to that runtime, so both see the same device allocations.
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise HataError(f"{LIB_PATH} is not built; run paper_2506_02572_amd/build.py")
        from . import build as _build
        _build.build(force=True)
    lib = ctypes.CDLL(LIB_PATH)
    lib.hata_strerror.restype = ctypes.c_char_p
    lib.hata_strerror.argtypes = [ctypes.c_int]
    lib.hata_workspace_bytes.argtypes = [ctypes.POINTER(hata_config), ctypes.POINTER(ctypes.c_size_t)]
    lib.hata_create.argtypes = [ctypes.POINTER(_vp), ctypes.POINTER(hata_config), _vp, ctypes.c_size_t]
    lib.hata_workspace_bytes_tuned.argtypes = [ctypes.POINTER(hata_config), ctypes.POINTER(hata_tuning),
                                               ctypes.POINTER(ctypes.c_size_t)]
    lib.hata_create_tuned.argtypes = [ctypes.POINTER(_vp), ctypes.POINTER(hata_config), ctypes.POINTER(hata_tuning),
                                      _vp, ctypes.c_size_t]
    lib.hata_destroy.argtypes = [_vp]
    lib.hata_encode_keys.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp]
    lib.hata_prepare_weights.argtypes = [_vp, _vp, _vp]
    lib.hata_prefill_write.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp]
    lib.hata_prefill_write_paged.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _i32,
                                             _i32, _i32, _vp, _vp]
    lib.hata_encode_query.argtypes = [_vp, _vp, _vp, _i32, _vp, _vp]
    lib.hata_hamming_score.argtypes = [_vp, _vp, _vp, _vp, _i32, _vp, _vp]
    lib.hata_topk.argtypes = [_vp, _vp, _vp, _vp, _i32, _vp, _vp]
    lib.hata_sparse_decode.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i32, ctypes.c_float, _vp, _vp, _vp]
    lib.hata_sparse_decode_static.argtypes = [ctypes.POINTER(hata_config), _vp, _vp, _vp, _vp, _vp, _i32,
                                              ctypes.c_float, _vp, _vp, _vp]
    lib.hata_gather_rows.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp]
    lib.hata_dense_decode.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, ctypes.c_float, _vp, _vp, _vp]
    lib.hata_select_step.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp]
    lib.hata_decode_step.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32,
                                     ctypes.c_float, _vp, _vp, _vp]
    lib.hata_decode_step_paged.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _vp,
                                           _i32, _i32, ctypes.c_float, _vp, _vp, _vp]
    lib.hata_step_plan.argtypes = [_vp, _i32, ctypes.POINTER(_i32), ctypes.POINTER(_i32), ctypes.POINTER(_i32)]
    lib.hata_step_sub_batches.argtypes = [_vp, _i32, ctypes.POINTER(_i32)]
    lib.hata_set_step_mode.argtypes = [_vp, _i32]
    lib.hata_keep_step_scores.argtypes = [_vp, _i32]
    lib.hata_set_wait_limit.argtypes = [_vp, _i32]
    lib.hata_check.argtypes = [_vp, _vp]
    lib.hata_host_device_pointer.argtypes = [_vp, ctypes.POINTER(_vp)]
    lib.hata_step_buffers.argtypes = [_vp, ctypes.POINTER(_vp), ctypes.POINTER(_vp), ctypes.POINTER(_vp)]
    lib.hata_probe_mfma_stream.argtypes = [_vp, ctypes.c_size_t, _i32, _i32, _vp]
    for name in EXPORTS:
        if name != "hata_strerror":
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load_library().hata_strerror(int(status)).decode()


def _check(status: int, what: str) -> None:
    if status != 0:
        raise HataError(f"{what} failed: {strerror(status)} ({status})")


def _ptr(t):
    """Device pointer of a torch tensor (or None).  A pinned host tensor (KV cache kept in host
    memory) is passed by the device-side address of its mapping."""
    if t is None:
        return None
    if not t.is_cuda:
        if t.device.type == "cpu" and t.is_pinned():
            dev = ctypes.c_void_p()
            _check(load_library().hata_host_device_pointer(ctypes.c_void_p(t.data_ptr()), ctypes.byref(dev)),
                   "hata_host_device_pointer")
            return dev
        raise HataError("expected a device tensor (or a pinned host tensor)")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream=None):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


@dataclass
class Shape:
    B_max: int
    Hq: int
    Hkv: int
    d: int
    r: int
    L_cap: int
    k_max: int


class Context:
    """Owns a hata_ctx and the torch-allocated workspace it points into."""

    def __init__(self, B_max, Hq, Hkv, d, r, L_cap, k_max, kv_strides=None, device="cuda:0", chunk=0,
                 attn_rows=0, par_merge=-1, shared_device=False):
        import torch
        lib = load_library()
        if not torch.cuda.is_available():
            raise HataError("no GPU visible: the HATA path has no CPU fallback")
        self.shape = Shape(B_max, Hq, Hkv, d, r, L_cap, k_max)
        if kv_strides is None:
            kv_strides = (Hkv * L_cap * d, L_cap * d, d)
        self.cfg = hata_config(B_max, Hq, Hkv, d, r, L_cap, k_max, *kv_strides)
        self.tuning = hata_tuning(chunk, attn_rows, par_merge, 1 if shared_device else 0)
        nbytes = ctypes.c_size_t(0)
        _check(lib.hata_workspace_bytes_tuned(ctypes.byref(self.cfg), ctypes.byref(self.tuning), ctypes.byref(nbytes)),
               "hata_workspace_bytes_tuned")
        self.device = torch.device(device)
        self.workspace = torch.empty(nbytes.value + 256, dtype=torch.uint8, device=self.device)
        base = self.workspace.data_ptr()
        self._ws_ptr = (base + 255) // 256 * 256
        self._h = ctypes.c_void_p(None)
        with torch.cuda.device(self.device):
            _check(lib.hata_create_tuned(ctypes.byref(self._h), ctypes.byref(self.cfg), ctypes.byref(self.tuning),
                                         ctypes.c_void_p(self._ws_ptr), nbytes.value), "hata_create_tuned")
        self.workspace_bytes = nbytes.value

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            load_library().hata_destroy(self._h)
            self._h = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- entry points (same names as the C ABI) ----
    def hata_encode_keys(self, K, W_H, start, n_new, B, max_new, codes, stream=None):
        _check(load_library().hata_encode_keys(self._h, _ptr(K), _ptr(W_H), _ptr(start), _ptr(n_new),
                                               B, max_new, _ptr(codes), _stream(stream)),
               "hata_encode_keys")

    def hata_prepare_weights(self, W_H, stream=None):
        _check(load_library().hata_prepare_weights(self._h, _ptr(W_H), _stream(stream)), "hata_prepare_weights")

    def hata_prefill_write(self, K_new, V_new, start, n_new, B, max_new, K, V, codes, W_H, stream=None):
        _check(load_library().hata_prefill_write(self._h, _ptr(K_new), _ptr(V_new), _ptr(start), _ptr(n_new),
                                                 B, max_new, _ptr(K), _ptr(V), _ptr(codes), _ptr(W_H),
                                                 _stream(stream)), "hata_prefill_write")

    def hata_prefill_write_paged(self, K_new, V_new, start, n_new, B, max_new, K_pool, V_pool, codes_pool,
                                 block_table, max_blocks, page_rows, n_pages, W_H, stream=None):
        _check(load_library().hata_prefill_write_paged(
            self._h, _ptr(K_new), _ptr(V_new), _ptr(start), _ptr(n_new), B, max_new, _ptr(K_pool),
            _ptr(V_pool), _ptr(codes_pool), _ptr(block_table), max_blocks, page_rows, n_pages, _ptr(W_H),
            _stream(stream)), "hata_prefill_write_paged")

    def hata_encode_query(self, q, W_H, B, qcodes, stream=None):
        _check(load_library().hata_encode_query(self._h, _ptr(q), _ptr(W_H), B, _ptr(qcodes),
                                                _stream(stream)), "hata_encode_query")

    def hata_hamming_score(self, qcodes, codes, seq_len, B, scores, stream=None):
        _check(load_library().hata_hamming_score(self._h, _ptr(qcodes), _ptr(codes), _ptr(seq_len), B,
                                                 _ptr(scores), _stream(stream)), "hata_hamming_score")

    def hata_topk(self, scores, seq_len, k, B, idx, stream=None):
        _check(load_library().hata_topk(self._h, _ptr(scores), _ptr(seq_len), _ptr(k), B, _ptr(idx),
                                        _stream(stream)), "hata_topk")

    def hata_sparse_decode(self, q, K, V, idx, k, B, sm_scale, out, out_f32=None, stream=None):
        _check(load_library().hata_sparse_decode(self._h, _ptr(q), _ptr(K), _ptr(V), _ptr(idx), _ptr(k),
                                                 B, sm_scale, _ptr(out), _ptr(out_f32),
                                                 _stream(stream)), "hata_sparse_decode")

    def hata_sparse_decode_static(self, q, K, V, idx, k, B, sm_scale, out, out_f32=None, stream=None):
        """The allocation-free variant: uses this context's shape only, not its workspace."""
        _check(load_library().hata_sparse_decode_static(ctypes.byref(self.cfg), _ptr(q), _ptr(K), _ptr(V), _ptr(idx),
                                                        _ptr(k), B, sm_scale, _ptr(out), _ptr(out_f32),
                                                        _stream(stream)), "hata_sparse_decode_static")

    def hata_gather_rows(self, K, V, idx, k, B, max_workgroups, K_stage, V_stage, stream=None):
        _check(load_library().hata_gather_rows(self._h, _ptr(K), _ptr(V), _ptr(idx), _ptr(k), B, max_workgroups,
                                               _ptr(K_stage), _ptr(V_stage), _stream(stream)), "hata_gather_rows")

    def hata_dense_decode(self, q, K, V, seq_len, B, sm_scale, out, out_f32=None, stream=None):
        _check(load_library().hata_dense_decode(self._h, _ptr(q), _ptr(K), _ptr(V), _ptr(seq_len), B,
                                                sm_scale, _ptr(out), _ptr(out_f32), _stream(stream)),
               "hata_dense_decode")

    def hata_decode_step(self, q, K, V, W_H, codes, seq_len, k, B, append, sm_scale, out,
                         out_f32=None, stream=None):
        _check(load_library().hata_decode_step(self._h, _ptr(q), _ptr(K), _ptr(V), _ptr(W_H),
                                               _ptr(codes), _ptr(seq_len), _ptr(k), B,
                                               1 if append else 0, sm_scale, _ptr(out),
                                               _ptr(out_f32), _stream(stream)), "hata_decode_step")

    def hata_select_step(self, q, K, W_H, codes, seq_len, k, B, append, idx, stream=None):
        _check(load_library().hata_select_step(self._h, _ptr(q), _ptr(K), _ptr(W_H), _ptr(codes), _ptr(seq_len),
                                               _ptr(k), B, 1 if append else 0, _ptr(idx), _stream(stream)),
               "hata_select_step")

    def hata_decode_step_paged(self, q, K_pool, V_pool, W_H, codes_pool, block_table, max_blocks,
                               page_rows, n_pages, seq_len, k, B, append, sm_scale, out, out_f32=None,
                               stream=None):
        _check(load_library().hata_decode_step_paged(
            self._h, _ptr(q), _ptr(K_pool), _ptr(V_pool), _ptr(W_H), _ptr(codes_pool), _ptr(block_table),
            max_blocks, page_rows, n_pages, _ptr(seq_len), _ptr(k), B, 1 if append else 0, sm_scale,
            _ptr(out), _ptr(out_f32), _stream(stream)), "hata_decode_step_paged")

    def hata_step_plan(self, B):
        """(n_launches, chunk, n_chunks) of hata_decode_step for a batch of B sequences."""
        n, c, nc = _i32(0), _i32(0), _i32(0)
        _check(load_library().hata_step_plan(self._h, B, ctypes.byref(n), ctypes.byref(c),
                                             ctypes.byref(nc)), "hata_step_plan")
        return n.value, c.value, nc.value

    def hata_step_sub_batches(self, B):
        """Launches of the single-launch form for a batch of B (0: the three-launch form is used)."""
        n = _i32(0)
        _check(load_library().hata_step_sub_batches(self._h, B, ctypes.byref(n)), "hata_step_sub_batches")
        return n.value

    def hata_set_step_mode(self, mode):
        _check(load_library().hata_set_step_mode(self._h, mode), "hata_set_step_mode")

    def hata_keep_step_scores(self, keep):
        _check(load_library().hata_keep_step_scores(self._h, 1 if keep else 0), "hata_keep_step_scores")

    def hata_set_wait_limit(self, polls):
        _check(load_library().hata_set_wait_limit(self._h, polls), "hata_set_wait_limit")

    def hata_check(self, stream=None):
        _check(load_library().hata_check(self._h, _stream(stream)), "hata_check")

    def prepared(self, name, *args, stream=None):
        """Marshal the arguments of entry point ``name`` once and return a zero-argument callable
        that issues exactly that C call (for launch loops where per-call marshalling would
        dominate).  Tensor arguments must stay alive as long as the callable is used."""
        fn = getattr(load_library(), name)
        cargs = [self._h]
        for a in args:
            if a is None or hasattr(a, "data_ptr"):
                cargs.append(_ptr(a))
            elif isinstance(a, bool):
                cargs.append(1 if a else 0)
            else:
                cargs.append(a)
        cargs.append(_stream(stream))
        cargs = tuple(cargs)

        def call():
            rc = fn(*cargs)
            if rc != 0:
                _check(rc, name)
        return call

    def hata_step_buffers(self):
        """torch views (no copy) of the workspace regions hata_decode_step writes:
        (qcodes int32 [B_max,Hq,Wd], scores int16 [B_max,Hkv,L_cap], idx int32 [B_max,Hkv,k_max])."""
        import torch
        qc, sc, ix = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
        _check(load_library().hata_step_buffers(self._h, ctypes.byref(qc), ctypes.byref(sc),
                                                ctypes.byref(ix)), "hata_step_buffers")
        s = self.shape
        base = self.workspace.data_ptr()

        def view(ptr, nbytes, dtype, shape):
            off = ptr.value - base
            return self.workspace[off:off + nbytes].view(dtype).view(*shape)

        Wd = s.r // 32
        return (view(qc, s.B_max * s.Hq * Wd * 4, torch.int32, (s.B_max, s.Hq, Wd)),
                view(sc, s.B_max * s.Hkv * s.L_cap * 2, torch.int16, (s.B_max, s.Hkv, s.L_cap)),
                view(ix, s.B_max * s.Hkv * s.k_max * 4, torch.int32, (s.B_max, s.Hkv, s.k_max)))


def hata_probe_mfma_stream(buf, mfma_iters, mode, stream=None):
    """Diagnostic launch (see include/hata.h): mode bit 0 = matrix-core waves, bit 1 = streaming waves."""
    _check(load_library().hata_probe_mfma_stream(_ptr(buf), buf.numel() * buf.element_size(), int(mfma_iters),
                                                 int(mode), _stream(stream)), "hata_probe_mfma_stream")
