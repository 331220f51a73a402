"""ctypes front end of the CPU oracle (oracle/gram_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's CPU-baseline leg.  Nothing here touches the HIP library, and the
HIP binding never imports this module.

The functions compose the C routines in the order of Algorithm 1 of the
paper: unique items of the batch, encode once per unique item (Eq. 4), gather
to interaction positions, accumulate dL/dH per unique item (Eq. 6), encoder
weight gradient once per unique item (Eq. 7/9).  `e2e` is the per-interaction
baseline of Section 3.3.  All arithmetic is float64; `*_f32` helpers round once.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gram_oracle.c")
_LIB = os.path.join(_HERE, "libgram_oracle.so")

F32, BF16 = 0, 1
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", _LIB, _SRC])
    return _LIB


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        i32p, i64p, f32p, f64p, vp = (C.POINTER(C.c_int32), C.POINTER(C.c_int64),
                                      C.POINTER(C.c_float), C.POINTER(C.c_double), C.c_void_p)
        L.oracle_num_threads.restype = C.c_int
        L.oracle_set_num_threads.restype = C.c_int
        L.oracle_set_num_threads.argtypes = [C.c_int]
        for name in ("oracle_unique", "oracle_unique_brute"):
            f = getattr(L, name)
            f.restype = C.c_int64
            f.argtypes = [i32p, C.c_int64, C.c_int32, i32p, i32p, i32p]
        L.oracle_encode.restype = C.c_int
        L.oracle_encode.argtypes = [i32p, C.c_int64, C.c_int32, C.c_int32, vp, vp, C.c_int,
                                    C.c_int32, C.c_int32, f64p]
        L.oracle_gather.restype = C.c_int
        L.oracle_gather.argtypes = [f64p, i32p, C.c_int64, C.c_int32, f64p]
        L.oracle_grad_accumulate.restype = C.c_int
        L.oracle_grad_accumulate.argtypes = [f32p, i32p, C.c_int64, i32p, C.c_int64, C.c_int32,
                                             C.c_int32, f64p]
        L.oracle_wgrad.restype = C.c_int
        L.oracle_wgrad.argtypes = [i32p, C.c_int64, C.c_int32, C.c_int32, vp, C.c_int, C.c_int32,
                                   C.c_int32, f64p, f64p]
        L.oracle_wgrad_entries.restype = C.c_int
        L.oracle_wgrad_entries.argtypes = [i32p, C.c_int64, C.c_int32, C.c_int32, vp, C.c_int,
                                           C.c_int32, C.c_int32, f64p, i32p, i32p, C.c_int64, f64p]
        L.oracle_buffer_new.restype = vp
        L.oracle_buffer_new.argtypes = [C.c_int32]
        L.oracle_buffer_free.restype = None
        L.oracle_buffer_free.argtypes = [vp]
        L.oracle_buffer_size.restype = C.c_int64
        L.oracle_buffer_size.argtypes = [vp]
        L.oracle_buffer_add.restype = C.c_int
        L.oracle_buffer_add.argtypes = [vp, i32p, i32p, f64p, C.c_int64]
        L.oracle_mlp_encode.restype = C.c_int
        L.oracle_mlp_encode.argtypes = [i32p, C.c_int64, C.c_int32, C.c_int32, vp, vp, vp, C.c_int, C.c_int32,
                                        C.c_int32, C.c_int32, f64p, f64p]
        L.oracle_mlp_grad.restype = C.c_int
        L.oracle_mlp_grad.argtypes = [i32p, C.c_int64, C.c_int32, C.c_int32, vp, vp, vp, C.c_int, C.c_int32,
                                      C.c_int32, C.c_int32, f64p, f64p, f64p]
        L.oracle_mlp_grad_entries.restype = C.c_int
        L.oracle_mlp_grad_entries.argtypes = [i32p, C.c_int64, C.c_int32, C.c_int32, vp, vp, vp, C.c_int, C.c_int32,
                                              C.c_int32, C.c_int32, f64p, i32p, i32p, C.c_int64, f64p, i32p, i32p,
                                              C.c_int64, f64p]
        L.oracle_buffer_add64.restype = C.c_int
        L.oracle_buffer_add64.argtypes = [vp, i32p, i64p, f64p, C.c_int64]
        L.oracle_buffer_export.restype = C.c_int
        L.oracle_buffer_export.argtypes = [vp, i32p, i64p, f64p]
        L.oracle_buffer_rows.restype = C.c_int
        L.oracle_buffer_rows.argtypes = [vp, i32p, C.c_int64, f64p]
        L.oracle_pseudo_target.restype = C.c_int
        L.oracle_pseudo_target.argtypes = [f64p, f64p, C.c_int64, C.c_int32, f64p, f64p]
        L.oracle_pseudo_loss_grad.restype = C.c_int
        L.oracle_pseudo_loss_grad.argtypes = [i32p, C.c_int64, C.c_int32, C.c_int32, vp, vp, C.c_int,
                                              C.c_int32, C.c_int32, f64p, f64p, f64p, f64p]
        _lib = L
    return _lib


class OracleError(RuntimeError):
    pass


def _check(rc, what):
    if rc < 0:
        raise OracleError(f"{what}: " + {-1: "bad argument", -2: "id out of range"}.get(rc, str(rc)))
    return rc


def num_threads() -> int:
    return lib().oracle_num_threads()


def set_num_threads(n: int) -> int:
    """OpenMP threads for the calls that follow; returns the number in force."""
    return lib().oracle_set_num_threads(int(n))


def _xw_dtype(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"X/W must be float32 or uint16 (bf16 bits), got {a.dtype}")


def _unique(fn, ids, vocab_n):
    ids = np.ascontiguousarray(ids, dtype=np.int32).reshape(-1)
    m = ids.size
    cap = max(1, min(m, vocab_n))
    uniq = np.empty(cap, np.int32)
    counts = np.empty(cap, np.int32)
    inverse = np.empty(max(1, m), np.int32)
    u = _check(fn(_p(ids, C.c_int32), m, vocab_n, _p(uniq, C.c_int32), _p(inverse, C.c_int32),
                  _p(counts, C.c_int32)), "unique")
    return uniq[:u].copy(), inverse[:m].copy(), counts[:u].copy()


def unique(ids, vocab_n):
    """(uniq ascending, inverse, counts) of a batch of item IDs."""
    return _unique(lib().oracle_unique, ids, vocab_n)


def unique_brute(ids, vocab_n):
    return _unique(lib().oracle_unique_brute, ids, vocab_n)


def encode(item, X, W, pad_id):
    """float64 [len(item), d]: one encoder output per listed item (Eq. 4)."""
    item = np.ascontiguousarray(item, dtype=np.int32).reshape(-1)
    X = np.ascontiguousarray(X)
    W = np.ascontiguousarray(W)
    dt = _xw_dtype(X)
    assert _xw_dtype(W) == dt and X.shape[1] == W.shape[0]
    d_in, d = W.shape
    E = np.empty((item.size, d), np.float64)
    _check(lib().oracle_encode(_p(item, C.c_int32), item.size, X.shape[0], pad_id,
                               X.ctypes.data, W.ctypes.data, dt, d_in, d, _p(E, C.c_double)), "encode")
    return E


def gather(E, inverse):
    E = np.ascontiguousarray(E, dtype=np.float64)
    inverse = np.ascontiguousarray(inverse, dtype=np.int32).reshape(-1)
    H = np.empty((inverse.size, E.shape[1]), np.float64)
    lib().oracle_gather(_p(E, C.c_double), _p(inverse, C.c_int32), inverse.size, E.shape[1],
                        _p(H, C.c_double))
    return H


def grad_accumulate(dH, inverse, uniq, pad_id, G=None):
    """float64 [U, d]: per-unique-item sum of dL/dH (Eq. 6); added to G if given."""
    dH = np.ascontiguousarray(dH, dtype=np.float32)
    inverse = np.ascontiguousarray(inverse, dtype=np.int32).reshape(-1)
    uniq = np.ascontiguousarray(uniq, dtype=np.int32)
    d = dH.shape[-1]
    dH = dH.reshape(-1, d)
    assert dH.shape[0] == inverse.size
    if G is None:
        G = np.zeros((uniq.size, d), np.float64)
    _check(lib().oracle_grad_accumulate(_p(dH, C.c_float), _p(inverse, C.c_int32), inverse.size,
                                        _p(uniq, C.c_int32), uniq.size, pad_id, d,
                                        _p(G, C.c_double)), "grad_accumulate")
    return G


def wgrad(item, X, G, pad_id):
    """float64 [d_in, d]: sum over listed items of X[item]^T (outer) G[row]."""
    item = np.ascontiguousarray(item, dtype=np.int32).reshape(-1)
    X = np.ascontiguousarray(X)
    G = np.ascontiguousarray(G, dtype=np.float64)
    assert G.shape[0] == item.size
    d_in, d = X.shape[1], G.shape[1]
    dW = np.empty((d_in, d), np.float64)
    _check(lib().oracle_wgrad(_p(item, C.c_int32), item.size, X.shape[0], pad_id, X.ctypes.data,
                              _xw_dtype(X), d_in, d, _p(G, C.c_double), _p(dW, C.c_double)), "wgrad")
    return dW


def wgrad_entries(item, X, G, pad_id, rows, cols):
    """float64 [n]: dW[rows[t], cols[t]] without forming dW."""
    item = np.ascontiguousarray(item, dtype=np.int32).reshape(-1)
    X = np.ascontiguousarray(X)
    G = np.ascontiguousarray(G, dtype=np.float64)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    cols = np.ascontiguousarray(cols, dtype=np.int32)
    out = np.empty(rows.size, np.float64)
    _check(lib().oracle_wgrad_entries(_p(item, C.c_int32), item.size, X.shape[0], pad_id,
                                      X.ctypes.data, _xw_dtype(X), X.shape[1], G.shape[1],
                                      _p(G, C.c_double), _p(rows, C.c_int32), _p(cols, C.c_int32),
                                      rows.size, _p(out, C.c_double)), "wgrad_entries")
    return out


def pseudo_target(E, G):
    """Pseudo-targets of Algorithm 1 step 3 (Eq. 6), h~ = h - grad L(h), and the pseudo-loss of
    Eq. 7 at the current encoder.  E, G: [U, d] float64 (G = the gradient accumulated for each
    item).  Returns (Ht [U, d] float64, loss)."""
    E = np.ascontiguousarray(E, dtype=np.float64)
    G = np.ascontiguousarray(G, dtype=np.float64)
    assert E.shape == G.shape and E.ndim == 2
    Ht = np.empty_like(E)
    loss = C.c_double(0.0)
    _check(lib().oracle_pseudo_target(_p(E, C.c_double), _p(G, C.c_double), E.shape[0], E.shape[1],
                                      _p(Ht, C.c_double), C.byref(loss)), "pseudo_target")
    return Ht, loss.value


def pseudo_loss_grad(item, X, W, Ht, pad_id=0):
    """One content-encoder batch of Algorithm 1 step 4: pseudo-loss of Eq. 7 for the listed items
    at the CURRENT weights W against stored pseudo-targets Ht [n, d], and its gradient.
    Returns float64 (miss [n, d] = X[item].W - Ht, loss, dW [d_in, d])."""
    item = np.ascontiguousarray(item, dtype=np.int32).reshape(-1)
    X = np.ascontiguousarray(X)
    W = np.ascontiguousarray(W)
    Ht = np.ascontiguousarray(Ht, dtype=np.float64)
    dt = _xw_dtype(X)
    assert _xw_dtype(W) == dt and X.shape[1] == W.shape[0]
    d_in, d = W.shape
    assert Ht.shape == (item.size, d)
    miss = np.empty((item.size, d), np.float64)
    dW = np.empty((d_in, d), np.float64)
    loss = C.c_double(0.0)
    _check(lib().oracle_pseudo_loss_grad(_p(item, C.c_int32), item.size, X.shape[0], pad_id,
                                         X.ctypes.data, W.ctypes.data, dt, d_in, d, _p(Ht, C.c_double),
                                         _p(miss, C.c_double), C.byref(loss), _p(dW, C.c_double)),
           "pseudo_loss_grad")
    return miss, loss.value, dW


def _mlp_args(item, X, W1, W2):
    item = np.ascontiguousarray(item, dtype=np.int32).reshape(-1)
    X, W1, W2 = np.ascontiguousarray(X), np.ascontiguousarray(W1), np.ascontiguousarray(W2)
    dt = _xw_dtype(X)
    assert _xw_dtype(W1) == dt and _xw_dtype(W2) == dt
    assert X.shape[1] == W1.shape[0] and W1.shape[1] == W2.shape[0]
    return item, X, W1, W2, dt


def mlp_encode(item, X, W1, W2, pad_id=0):
    """Two-layer stand-in encoder, h = max(x.W1, 0).W2, once per listed item.
    Returns float64 (A1 [n, d_hid] hidden activations, E [n, d])."""
    item, X, W1, W2, dt = _mlp_args(item, X, W1, W2)
    (d_in, d_hid), d = W1.shape, W2.shape[1]
    A1 = np.empty((item.size, d_hid), np.float64)
    E = np.empty((item.size, d), np.float64)
    _check(lib().oracle_mlp_encode(_p(item, C.c_int32), item.size, X.shape[0], pad_id, X.ctypes.data,
                                   W1.ctypes.data, W2.ctypes.data, dt, d_in, d_hid, d,
                                   _p(A1, C.c_double), _p(E, C.c_double)), "mlp_encode")
    return A1, E


def mlp_grad(item, X, W1, W2, R, pad_id=0):
    """Backward pass of the two-layer encoder for the listed items given dL/dh rows R [n, d].
    Returns float64 (dW1 [d_in, d_hid], dW2 [d_hid, d])."""
    item, X, W1, W2, dt = _mlp_args(item, X, W1, W2)
    (d_in, d_hid), d = W1.shape, W2.shape[1]
    R = np.ascontiguousarray(R, dtype=np.float64)
    assert R.shape == (item.size, d)
    dW1 = np.empty((d_in, d_hid), np.float64)
    dW2 = np.empty((d_hid, d), np.float64)
    _check(lib().oracle_mlp_grad(_p(item, C.c_int32), item.size, X.shape[0], pad_id, X.ctypes.data,
                                 W1.ctypes.data, W2.ctypes.data, dt, d_in, d_hid, d, _p(R, C.c_double),
                                 _p(dW1, C.c_double), _p(dW2, C.c_double)), "mlp_grad")
    return dW1, dW2


def mlp_grad_entries(item, X, W1, W2, R, i1, q1, q2, c2, pad_id=0):
    """float64 (dW1[i1[t], q1[t]], dW2[q2[t], c2[t]]) of mlp_grad without forming the matrices."""
    item, X, W1, W2, dt = _mlp_args(item, X, W1, W2)
    (d_in, d_hid), d = W1.shape, W2.shape[1]
    R = np.ascontiguousarray(R, dtype=np.float64)
    assert R.shape == (item.size, d)
    i1, q1, q2, c2 = (np.ascontiguousarray(a, dtype=np.int32) for a in (i1, q1, q2, c2))
    out1, out2 = np.empty(i1.size, np.float64), np.empty(q2.size, np.float64)
    _check(lib().oracle_mlp_grad_entries(_p(item, C.c_int32), item.size, X.shape[0], pad_id, X.ctypes.data,
                                         W1.ctypes.data, W2.ctypes.data, dt, d_in, d_hid, d, _p(R, C.c_double),
                                         _p(i1, C.c_int32), _p(q1, C.c_int32), i1.size, _p(out1, C.c_double),
                                         _p(q2, C.c_int32), _p(c2, C.c_int32), q2.size, _p(out2, C.c_double)),
           "mlp_grad_entries")
    return out1, out2


def mlp_e2e(ids, X, W1, W2, dH, pad_id=0):
    """End-to-end baseline with the two-layer encoder: forward and backward once per interaction
    (Section 3.3).  Returns float64 (H [M, d], dW1, dW2)."""
    ids = np.ascontiguousarray(ids, dtype=np.int32).reshape(-1)
    d = W2.shape[1]
    _, H = mlp_encode(ids, X, W1, W2, pad_id)
    dW1, dW2 = mlp_grad(ids, X, W1, W2, np.asarray(dH, np.float32).reshape(-1, d).astype(np.float64), pad_id)
    return H, dW1, dW2


def mlp_gram_single(ids, X, W1, W2, dH, pad_id=0):
    """Single-step GRAM with the two-layer encoder: encode, keep activations and back-propagate
    once per unique item (Algorithm 1 with N = 1)."""
    ids = np.ascontiguousarray(ids, dtype=np.int32).reshape(-1)
    uniq, inverse, counts = unique(ids, X.shape[0])
    A1, E = mlp_encode(uniq, X, W1, W2, pad_id)
    H = gather(E, inverse)
    G = grad_accumulate(dH, inverse, uniq, pad_id)
    dW1, dW2 = mlp_grad(uniq, X, W1, W2, G, pad_id)
    return dict(uniq=uniq, inverse=inverse, counts=counts, A1=A1, E=E, H=H, G=G, dW1=dW1, dW2=dW2)


def mlp_pseudo_loss_grad(item, X, W1, W2, Ht, pad_id=0):
    """One content-encoder batch of Algorithm 1 step 4 with the two-layer encoder: miss = h - Ht at the
    current weights (zero for padding), pseudo-loss of Eq. 7, and its gradients.
    Returns float64 (miss, loss, dW1, dW2)."""
    item = np.ascontiguousarray(item, dtype=np.int32).reshape(-1)
    _, E = mlp_encode(item, X, W1, W2, pad_id)
    miss = E - np.ascontiguousarray(Ht, dtype=np.float64)
    miss[item == pad_id] = 0.0
    dW1, dW2 = mlp_grad(item, X, W1, W2, miss, pad_id)
    return miss, 0.5 * float(np.sum(miss * miss)), dW1, dW2


def e2e(ids, X, W, dH, pad_id=0):
    """End-to-end baseline (Section 3.3): the encoder runs forward and backward
    once per interaction.  Returns float64 (H [M,d], dW [d_in,d])."""
    ids = np.ascontiguousarray(ids, dtype=np.int32).reshape(-1)
    d = W.shape[1]
    H = encode(ids, X, W, pad_id)
    dW = wgrad(ids, X, np.asarray(dH, dtype=np.float32).reshape(-1, d).astype(np.float64), pad_id)
    return H, dW


def gram_single(ids, X, W, dH, pad_id=0):
    """Single-step GRAM (Section 4.1; Algorithm 1 with N = 1), float64 results."""
    ids = np.ascontiguousarray(ids, dtype=np.int32).reshape(-1)
    uniq, inverse, counts = unique(ids, X.shape[0])
    E = encode(uniq, X, W, pad_id)
    H = gather(E, inverse)
    G = grad_accumulate(dH, inverse, uniq, pad_id)
    dW = wgrad(uniq, X, G, pad_id)
    return dict(uniq=uniq, inverse=inverse, counts=counts, E=E, H=H, G=G, dW=dW)


class GramMulti:
    """Multi-step GRAM (Section 4.2): the gradient buffer persists over the N
    mini-batches of a window; one weight gradient at its end."""

    def __init__(self, X, W, pad_id=0):
        self.X, self.W, self.pad_id = np.ascontiguousarray(X), np.ascontiguousarray(W), pad_id
        self.d = self.W.shape[1]
        self._buf = lib().oracle_buffer_new(self.d)
        self.steps = 0

    def step(self, ids, dH):
        """One mini-batch: returns this step's dict(uniq, inverse, counts, E, H, G)."""
        ids = np.ascontiguousarray(ids, dtype=np.int32).reshape(-1)
        uniq, inverse, counts = unique(ids, self.X.shape[0])
        E = encode(uniq, self.X, self.W, self.pad_id)
        H = gather(E, inverse)
        G = grad_accumulate(dH, inverse, uniq, self.pad_id)
        _check(lib().oracle_buffer_add(self._buf, _p(uniq, C.c_int32), _p(counts, C.c_int32),
                                       _p(G, C.c_double), uniq.size), "buffer_add")
        self.steps += 1
        return dict(uniq=uniq, inverse=inverse, counts=counts, E=E, H=H, G=G)

    def resume(self, ids, counts, G):
        """Merge a saved window state (ids ascending, 64-bit counts, gradient rows) into the
        buffer: a window interrupted after some steps and resumed gives the uninterrupted result."""
        ids = np.ascontiguousarray(ids, dtype=np.int32).reshape(-1)
        counts = np.ascontiguousarray(counts, dtype=np.int64).reshape(-1)
        G = np.ascontiguousarray(G, dtype=np.float64).reshape(ids.size, self.d)
        assert counts.size == ids.size and np.all(np.diff(ids) > 0)
        _check(lib().oracle_buffer_add64(self._buf, _p(ids, C.c_int32), _p(counts, C.c_int64),
                                         _p(G, C.c_double), ids.size), "buffer_add64")

    def rows(self, ids):
        """Gradient accumulated so far in the window for each of `ids` (zeros if absent)."""
        ids = np.ascontiguousarray(ids, dtype=np.int32).reshape(-1)
        G = np.empty((ids.size, self.d), np.float64)
        _check(lib().oracle_buffer_rows(self._buf, _p(ids, C.c_int32), ids.size, _p(G, C.c_double)),
               "buffer_rows")
        return G

    def export(self):
        n = lib().oracle_buffer_size(self._buf)
        ids = np.empty(n, np.int32)
        counts = np.empty(n, np.int64)
        G = np.empty((n, self.d), np.float64)
        lib().oracle_buffer_export(self._buf, _p(ids, C.c_int32), _p(counts, C.c_int64),
                                   _p(G, C.c_double))
        return ids, counts, G

    def finish(self, full_dw=True):
        """End of the window: (uniq_tot, counts_tot, G_tot, dW) and an empty buffer."""
        ids, counts, G = self.export()
        dW = wgrad(ids, self.X, G, self.pad_id) if full_dw else None
        lib().oracle_buffer_free(self._buf)
        self._buf = lib().oracle_buffer_new(self.d)
        self.steps = 0
        return dict(uniq=ids, counts=counts, G=G, dW=dW)

    def __del__(self):
        try:
            lib().oracle_buffer_free(self._buf)
        except Exception:
            pass


def boost_ratio(ids, pad_id=0):
    """R of Eq. 10: interactions in the batch / unique items in the batch
    (padding is neither an interaction nor an item)."""
    ids = np.ascontiguousarray(ids, dtype=np.int32).reshape(-1)
    uniq, _, counts = unique(ids, int(ids.max()) + 1 if ids.size else 1)
    keep = uniq != pad_id
    return int(counts[keep].sum()) / max(1, int(keep.sum()))
