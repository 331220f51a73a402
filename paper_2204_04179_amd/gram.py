"""Thin ctypes binding of libgram (include/gram.h).

Argument marshalling only: every step of the path runs in the HIP kernels of
the library.  PyTorch supplies device memory and the current stream.  There is
no fallback: if the shared library is missing or fails to load, `load()`
raises.
"""
from __future__ import annotations

import ctypes as C
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libgram.so")

F32, BF16 = 0, 1
OK, ERR_ARG, ERR_CAPACITY, ERR_SEQUENCE, ERR_RANGE, ERR_HIP, ERR_UNIMPLEMENTED = 0, -1, -2, -3, -4, -5, -6
STATUS_NAMES = {OK: "GRAM_OK", ERR_ARG: "GRAM_ERR_ARG", ERR_CAPACITY: "GRAM_ERR_CAPACITY",
                ERR_SEQUENCE: "GRAM_ERR_SEQUENCE", ERR_RANGE: "GRAM_ERR_RANGE", ERR_HIP: "GRAM_ERR_HIP",
                ERR_UNIMPLEMENTED: "GRAM_ERR_UNIMPLEMENTED"}

EXPORTS = ("gram_workspace_bytes", "gram_create", "gram_destroy", "gram_unique", "gram_encode_gather",
           "gram_grad_accumulate", "gram_pseudo_target", "gram_gather", "gram_encoder_wgrad",
           "gram_encoder_wgrad_chunk", "gram_pseudo_loss_grad", "gram_flush",
           "gram_flush64", "gram_window_end", "gram_window_import", "gram_mlp_encode_gather", "gram_mlp_batch_bytes",
           "gram_mlp_backward", "gram_unique_static",
           "gram_check", "gram_last_error",
           "gram_kernel_count", "gram_kernel_name", "gram_light_max", "gram_profile_enable",
           "gram_profile_read")


class GramConfig(C.Structure):
    _fields_ = [("vocab_n", C.c_int32), ("d_in", C.c_int32), ("d", C.c_int32),
                ("max_positions", C.c_int64), ("k_steps", C.c_int32), ("pad_id", C.c_int32),
                ("u_total_cap", C.c_int64), ("xw_dtype", C.c_int32), ("buffer_layout", C.c_int32),
                ("d_hidden", C.c_int32), ("h_dtype", C.c_int32)]


class GramError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


_lib = None


def load():
    """Open libgram.so (built by `python -m paper_2204_04179_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2204_04179_amd.build`")
    # PyTorch ships a HIP runtime of its own.  It has to be in the process before this library is
    # opened, so that the library binds to the same runtime as the tensors it is handed; opened
    # the other way round, PyTorch finds no device afterwards.
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    vp, i32p = C.c_void_p, C.POINTER(C.c_int32)
    L.gram_workspace_bytes.restype = C.c_int64
    L.gram_workspace_bytes.argtypes = [C.POINTER(GramConfig)]
    L.gram_create.restype = C.c_int
    L.gram_create.argtypes = [C.POINTER(vp), C.POINTER(GramConfig)]
    L.gram_destroy.restype = C.c_int
    L.gram_destroy.argtypes = [vp]
    L.gram_unique.restype = C.c_int
    L.gram_unique.argtypes = [vp, vp, C.c_int64, vp, vp, vp, vp, i32p, vp]
    L.gram_encode_gather.restype = C.c_int
    L.gram_encode_gather.argtypes = [vp, vp, vp, vp, vp, vp, C.c_int64, vp, vp, vp]
    L.gram_grad_accumulate.restype = C.c_int
    L.gram_grad_accumulate.argtypes = [vp, vp, C.c_int64, C.c_int32, vp]
    L.gram_encoder_wgrad_chunk.restype = C.c_int
    L.gram_encoder_wgrad_chunk.argtypes = [vp, vp, vp, C.c_int64, C.c_int64, C.c_int32, vp]
    L.gram_pseudo_loss_grad.restype = C.c_int
    L.gram_pseudo_loss_grad.argtypes = [vp, vp, vp, vp, vp, C.c_int64, vp, vp, C.c_int32, vp, vp]
    L.gram_pseudo_target.restype = C.c_int
    L.gram_pseudo_target.argtypes = [vp, vp, vp, vp, vp]
    L.gram_gather.restype = C.c_int
    L.gram_gather.argtypes = [vp, vp, vp, C.c_int64, vp, vp]
    L.gram_encoder_wgrad.restype = C.c_int
    L.gram_encoder_wgrad.argtypes = [vp, vp, vp, vp]
    L.gram_flush.restype = C.c_int
    L.gram_flush.argtypes = [vp, vp, vp, vp, vp, i32p, vp]
    L.gram_window_end.restype = C.c_int
    L.gram_window_end.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32p, vp]
    L.gram_mlp_encode_gather.restype = C.c_int
    L.gram_mlp_encode_gather.argtypes = [vp, vp, vp, vp, vp, vp, vp, C.c_int64, vp, vp, vp, vp]
    L.gram_mlp_batch_bytes.restype = C.c_int64
    L.gram_mlp_batch_bytes.argtypes = [vp, C.c_int64]
    L.gram_mlp_backward.restype = C.c_int
    L.gram_mlp_backward.argtypes = [vp, vp, vp, vp, vp, vp, vp, C.c_int64, vp, vp, vp, C.c_int32, vp, vp]
    L.gram_flush64.restype = C.c_int
    L.gram_flush64.argtypes = [vp, vp, vp, vp, vp, i32p, vp]
    L.gram_window_import.restype = C.c_int
    L.gram_window_import.argtypes = [vp, vp, vp, vp, C.c_int64, vp]
    L.gram_unique_static.restype = C.c_int
    L.gram_unique_static.argtypes = [vp, C.c_int64, C.c_int32, C.c_int32, vp, vp, vp, vp, vp, vp]
    L.gram_check.restype = C.c_int
    L.gram_check.argtypes = [vp, vp]
    L.gram_last_error.restype = C.c_char_p
    L.gram_last_error.argtypes = [vp]
    L.gram_kernel_count.restype = C.c_int
    L.gram_kernel_count.argtypes = []
    L.gram_light_max.restype = C.c_int
    L.gram_light_max.argtypes = []
    L.gram_kernel_name.restype = C.c_char_p
    L.gram_kernel_name.argtypes = [C.c_int]
    L.gram_profile_enable.restype = C.c_int
    L.gram_profile_enable.argtypes = [vp, C.c_uint64, C.c_int32]
    L.gram_profile_read.restype = C.c_int
    L.gram_profile_read.argtypes = [vp, C.c_int, C.POINTER(C.c_int64), C.POINTER(C.c_double)]
    _lib = L
    return L


def make_config(vocab_n, d_in, d, max_positions, k_steps=1, pad_id=0, u_total_cap=0, xw_dtype=BF16,
                buffer_layout=0, d_hidden=0, h_dtype=F32):
    return GramConfig(int(vocab_n), int(d_in), int(d), int(max_positions), int(k_steps), int(pad_id),
                      int(u_total_cap), int(xw_dtype), int(buffer_layout), int(d_hidden), int(h_dtype))


def workspace_bytes(cfg: GramConfig) -> int:
    return load().gram_workspace_bytes(C.byref(cfg))


def _ptr(t):
    """Device (or NULL) pointer of a torch tensor / raw int."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


UNIQUE_STATIC_MAX_POSITIONS = 262144


def unique_static(ids, vocab_n, pad_id, uniq, inverse, counts, u_dev, err_dev=None, m=None, stream=None):
    """gram_unique_static: the dedup step without a context and without any allocation."""
    L = load()
    rc = L.gram_unique_static(_ptr(ids), int(ids.numel() if m is None else m), int(vocab_n), int(pad_id),
                              _ptr(uniq), _ptr(inverse), _ptr(counts), _ptr(u_dev), _ptr(err_dev),
                              _stream(stream))
    if rc != OK:
        raise GramError(rc, (L.gram_last_error(None) or b"").decode())


class Gram:
    """A context of the library.  Tensor arguments are CUDA(HIP) torch tensors,
    contiguous, of the dtypes include/gram.h states; they are passed by pointer."""

    def __init__(self, cfg: GramConfig):
        self._lib = load()
        self.cfg = cfg
        self._h = C.c_void_p()
        rc = self._lib.gram_create(C.byref(self._h), C.byref(cfg))
        if rc != OK:
            raise GramError(rc, (self._lib.gram_last_error(None) or b"").decode())

    def _ck(self, rc):
        if rc != OK:
            raise GramError(rc, (self._lib.gram_last_error(self._h) or b"").decode())

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            self._lib.gram_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def unique(self, ids, uniq, inverse, counts, u_dev=None, want_host_u=False, stream=None):
        m = ids.numel() if not isinstance(ids, int) else None
        u_host = C.c_int32(-1)
        self._ck(self._lib.gram_unique(self._h, _ptr(ids), m, _ptr(uniq), _ptr(inverse), _ptr(counts),
                                       _ptr(u_dev), C.byref(u_host) if want_host_u else None,
                                       _stream(stream)))
        return u_host.value if want_host_u else None

    def encode_gather(self, X, W, uniq, inverse, u_dev, m, E, H, stream=None):
        self._ck(self._lib.gram_encode_gather(self._h, _ptr(X), _ptr(W), _ptr(uniq), _ptr(inverse),
                                              _ptr(u_dev), int(m), _ptr(E), _ptr(H), _stream(stream)))

    def grad_accumulate(self, dH, m, step_k, stream=None):
        self._ck(self._lib.gram_grad_accumulate(self._h, _ptr(dH), int(m), int(step_k), _stream(stream)))

    def pseudo_target(self, E, Ht=None, loss_dev=None, stream=None):
        self._ck(self._lib.gram_pseudo_target(self._h, _ptr(E), _ptr(Ht), _ptr(loss_dev), _stream(stream)))

    def gather(self, src, inverse, m, H, stream=None):
        self._ck(self._lib.gram_gather(self._h, _ptr(src), _ptr(inverse), int(m), _ptr(H), _stream(stream)))

    def encoder_wgrad(self, X, dW, stream=None):
        self._ck(self._lib.gram_encoder_wgrad(self._h, _ptr(X), _ptr(dW), _stream(stream)))

    def encoder_wgrad_chunk(self, X, dW, first_row, n_rows, accumulate, stream=None):
        self._ck(self._lib.gram_encoder_wgrad_chunk(self._h, _ptr(X), _ptr(dW), int(first_row), int(n_rows),
                                                    1 if accumulate else 0, _stream(stream)))

    def pseudo_loss_grad(self, X, W, ids, Ht, n, R, dW, accumulate=False, loss_dev=None, stream=None):
        self._ck(self._lib.gram_pseudo_loss_grad(self._h, _ptr(X), _ptr(W), _ptr(ids), _ptr(Ht), int(n),
                                                 _ptr(R), _ptr(dW), 1 if accumulate else 0,
                                                 _ptr(loss_dev), _stream(stream)))

    def flush(self, uniq_total=None, counts_total=None, G_total=None, u_total_dev=None,
              want_host_u=False, stream=None):
        u_host = C.c_int32(-1)
        self._ck(self._lib.gram_flush(self._h, _ptr(uniq_total), _ptr(counts_total), _ptr(G_total),
                                      _ptr(u_total_dev), C.byref(u_host) if want_host_u else None,
                                      _stream(stream)))
        return u_host.value if want_host_u else None

    def window_end(self, X, dW, uniq_total=None, counts_total=None, G_total=None, u_total_dev=None,
                   want_host_u=False, stream=None):
        u_host = C.c_int32(-1)
        self._ck(self._lib.gram_window_end(self._h, _ptr(X), _ptr(dW), _ptr(uniq_total), _ptr(counts_total),
                                           _ptr(G_total), _ptr(u_total_dev),
                                           C.byref(u_host) if want_host_u else None, _stream(stream)))
        return u_host.value if want_host_u else None

    def mlp_encode_gather(self, X, W1, W2, uniq, inverse, u_dev, m, A1, E, H, stream=None):
        self._ck(self._lib.gram_mlp_encode_gather(self._h, _ptr(X), _ptr(W1), _ptr(W2), _ptr(uniq), _ptr(inverse),
                                                  _ptr(u_dev), int(m), _ptr(A1), _ptr(E), _ptr(H),
                                                  _stream(stream)))

    def mlp_batch_bytes(self, n):
        return int(self._lib.gram_mlp_batch_bytes(self._h, int(n)))

    def mlp_backward(self, X, W1, W2, ids, G_rows, Ht, n, work, dW1, dW2, accumulate=False, loss_dev=None,
                     stream=None):
        self._ck(self._lib.gram_mlp_backward(self._h, _ptr(X), _ptr(W1), _ptr(W2), _ptr(ids), _ptr(G_rows),
                                             _ptr(Ht), int(n), _ptr(work), _ptr(dW1), _ptr(dW2),
                                             1 if accumulate else 0, _ptr(loss_dev), _stream(stream)))

    def flush64(self, uniq_total=None, counts_total=None, G_total=None, u_total_dev=None,
                want_host_u=False, stream=None):
        u_host = C.c_int32(-1)
        self._ck(self._lib.gram_flush64(self._h, _ptr(uniq_total), _ptr(counts_total), _ptr(G_total),
                                        _ptr(u_total_dev), C.byref(u_host) if want_host_u else None,
                                        _stream(stream)))
        return u_host.value if want_host_u else None

    def window_import(self, ids, counts, G_rows, n, stream=None):
        self._ck(self._lib.gram_window_import(self._h, _ptr(ids), _ptr(counts), _ptr(G_rows), int(n),
                                              _stream(stream)))

    def light_max(self):
        return int(self._lib.gram_light_max())

    def kernel_names(self):
        return [self._lib.gram_kernel_name(k).decode() for k in range(self._lib.gram_kernel_count())]

    def profile_enable(self, kernels=None, max_launches=8192):
        """Time the named kernels (all if None, none if empty) with HIP events."""
        names = self.kernel_names()
        mask = 0
        for k, nm in enumerate(names):
            if kernels is None or nm in kernels:
                mask |= 1 << k
        self._ck(self._lib.gram_profile_enable(self._h, mask, max_launches if mask else 0))

    def profile_read(self):
        """{kernel: (launches, total_ms)} of the timed launches so far."""
        out = {}
        for k, nm in enumerate(self.kernel_names()):
            n, ms = C.c_int64(0), C.c_double(0.0)
            self._ck(self._lib.gram_profile_read(self._h, k, C.byref(n), C.byref(ms)))
            if n.value:
                out[nm] = (n.value, ms.value)
        return out

    def check(self, stream=None):
        self._ck(self._lib.gram_check(self._h, _stream(stream)))
