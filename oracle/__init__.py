"""CPU oracle for the truly sparse MLP training step -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end of ``sparse_mlp_oracle.c`` (plain fp64-accumulating loops
over CSR, written from the operation definitions of Section 4 of the paper) plus
``mlp_step``, which strings the operations together in the order of the training loop
in the Appendix B listing: feedforward, loss gradient / batch size, backpropagate,
optimize.  Nothing here is imported by the HIP library or its binding; only tests, the
smoke check and the benchmark's CPU-baseline leg may use it.

All dense matrices are numpy arrays of shape (features, batch): one example per column.
``dtype`` is the storage type: float32 (what the GPU path stores) or float64 (finite
differences).  Every op returns the result and, where asked, the normaliser
S = sum of |terms| used by the parity metric  |candidate - oracle| <= tol * S.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sparse_mlp_oracle.c")
_LIB = os.path.join(_HERE, "libsparse_mlp_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no HIP, no BLAS)."""
    deps = [_SRC, os.path.join(_HERE, "sparse_mlp_oracle_impl.inc")]
    if (not force and os.path.exists(_LIB)
            and all(os.path.getmtime(_LIB) >= os.path.getmtime(d) for d in deps)):
        return _LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", _SRC, "-o", _LIB, "-lm"]
    subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(ctypes.c_int(n))


def _suffix(dtype) -> str:
    dtype = np.dtype(dtype)
    if dtype == np.float32:
        return "_f32"
    if dtype == np.float64:
        return "_f64"
    raise TypeError("oracle stores float32 or float64")


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _mat(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    assert a.ndim == 2
    return a


def _vec(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    assert a.ndim == 1
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


I32, I64, DBL = ctypes.c_int32, ctypes.c_int64, ctypes.c_double


def spmm(rows, cols, indptr, indices, values, bias, X, relu, dtype=np.float32, want_S=True):
    """Y = act(W X + b); returns (Y, S)."""
    X = _mat(X, dtype); B = X.shape[1]
    assert X.shape[0] == cols
    indptr, indices, values = _i32(indptr), _i32(indices), _vec(values, dtype)
    bias = None if bias is None else _vec(bias, dtype)
    Y = np.empty((rows, B), dtype=dtype)
    S = np.empty((rows, B), dtype=np.float64) if want_S else None
    getattr(_load(), "oracle_spmm" + _suffix(dtype))(
        I32(rows), I32(cols), _p(indptr), _p(indices), _p(values), _p(bias), _p(X), I64(B),
        I32(B), I32(1 if relu else 0), _p(Y), I64(B), _p(S))
    return Y, S


def spmm_t(rows, cols, indptr, indices, values, dZ, dtype=np.float32, want_S=True):
    """dX = W^T dZ; returns (dX, S)."""
    dZ = _mat(dZ, dtype); B = dZ.shape[1]
    assert dZ.shape[0] == rows
    indptr, indices, values = _i32(indptr), _i32(indices), _vec(values, dtype)
    dX = np.empty((cols, B), dtype=dtype)
    acc = np.empty((cols, B), dtype=np.float64)
    S = np.empty((cols, B), dtype=np.float64) if want_S else None
    getattr(_load(), "oracle_spmm_t" + _suffix(dtype))(
        I32(rows), I32(cols), _p(indptr), _p(indices), _p(values), _p(dZ), I64(B), I32(B),
        _p(dX), I64(B), _p(acc), _p(S))
    return dX, S


def relu_backward(dA, A, dtype=np.float32):
    dA, A = _mat(dA, dtype), _mat(A, dtype)
    assert dA.shape == A.shape
    n, B = A.shape
    dZ = np.empty((n, B), dtype=dtype)
    getattr(_load(), "oracle_relu_backward" + _suffix(dtype))(
        I32(n), I32(B), _p(dA), I64(B), _p(A), I64(B), _p(dZ), I64(B))
    return dZ


def sddmm(rows, cols, indptr, indices, dZ, X, dtype=np.float32, want_S=True):
    """g[p] = <dZ[row(p),:], X[indices[p],:]>, db = row sums of dZ; returns (g, Sg, db, Sdb)."""
    dZ, X = _mat(dZ, dtype), _mat(X, dtype)
    B = X.shape[1]
    assert dZ.shape == (rows, B) and X.shape[0] == cols
    indptr, indices = _i32(indptr), _i32(indices)
    nnz = int(indptr[-1])
    g = np.empty(nnz, dtype=dtype); db = np.empty(rows, dtype=dtype)
    Sg = np.empty(nnz, dtype=np.float64) if want_S else None
    Sdb = np.empty(rows, dtype=np.float64) if want_S else None
    getattr(_load(), "oracle_sddmm" + _suffix(dtype))(
        I32(rows), I32(cols), _p(indptr), _p(indices), _p(dZ), I64(B), _p(X), I64(B), I32(B),
        _p(g), _p(Sg), _p(db), _p(Sdb))
    return g, Sg, db, Sdb


def softmax_ce(Z, labels, dtype=np.float32, want_S=True):
    """Mean softmax cross-entropy of logits Z (classes, batch) and dZ = dloss/dZ.
    Returns (loss, S_loss, dZ, SdZ)."""
    Z = _mat(Z, dtype); labels = _i32(labels)
    rows, B = Z.shape
    assert labels.shape == (B,) and labels.min(initial=0) >= 0 and labels.max(initial=0) < rows
    dZ = np.empty((rows, B), dtype=dtype)
    SdZ = np.empty((rows, B), dtype=np.float64) if want_S else None
    out = np.zeros(2, dtype=np.float64)
    getattr(_load(), "oracle_softmax_ce" + _suffix(dtype))(
        I32(rows), I32(B), _p(Z), I64(B), _p(labels), _p(dZ), I64(B), _p(SdZ), _p(out))
    return float(out[0]), float(out[1]), dZ, SdZ


def momentum(w, v, g, lr, mu, Sg=None, dtype=np.float32, nesterov=False):
    """v <- mu v - lr g ; w <- w + v  (nesterov: w <- w + mu v_new - lr g).
    Returns new (w, v, Sw, Sv); inputs are not modified.
    For float32 storage lr and mu are first rounded to float32, as a float argument would be."""
    w = _vec(w, dtype).copy(); v = _vec(v, dtype).copy(); g = _vec(g, dtype)
    n = w.shape[0]
    assert v.shape == (n,) and g.shape == (n,)
    if np.dtype(dtype) == np.float32:
        lr, mu = float(np.float32(lr)), float(np.float32(mu))
    Sg = None if Sg is None else _vec(Sg, np.float64)
    Sv = np.empty(n, dtype=np.float64); Sw = np.empty(n, dtype=np.float64)
    getattr(_load(), "oracle_momentum" + _suffix(dtype))(
        I64(n), _p(w), _p(v), _p(g), DBL(lr), DBL(mu), I32(1 if nesterov else 0), _p(Sg), _p(Sv), _p(Sw))
    return w, v, Sw, Sv


# ---------------------------------------------------------------------------
# One training step of the static-sparse MLP
# ---------------------------------------------------------------------------

def new_state(layers, dtype=np.float32) -> List[Dict[str, np.ndarray]]:
    """Mutable per-layer state from workload layer records: values, bias and zero velocities.
    The pattern arrays are shared, never copied or written."""
    st = []
    for l in layers:
        st.append(dict(rows=l.rows, cols=l.cols, indptr=l.indptr, indices=l.indices, relu=l.relu,
                       values=np.array(l.values, dtype=dtype), bias=np.array(l.bias, dtype=dtype),
                       vel_w=np.zeros(l.nnz, dtype=dtype), vel_b=np.zeros(l.rows, dtype=dtype)))
    return st


def mlp_forward(state, X, dtype=np.float32, want_S=False):
    """Activations A_1..A_L (A_L = logits) and, if asked, their normalisers."""
    A, S = [], []
    a = np.ascontiguousarray(X, dtype=dtype)
    for l in state:
        a, s = spmm(l["rows"], l["cols"], l["indptr"], l["indices"], l["values"], l["bias"], a,
                    l["relu"], dtype, want_S)
        A.append(a); S.append(s)
    return A, S


def mlp_loss(state, X, labels, dtype=np.float64) -> float:
    A, _ = mlp_forward(state, X, dtype)
    return softmax_ce(A[-1], labels, dtype, want_S=False)[0]


def mlp_step(state, X, labels, lr, mu, dtype=np.float32, update=True,
             relu_masks: Optional[Sequence[Optional[np.ndarray]]] = None, nesterov=False):
    """One iteration of the training loop (Appendix B listing), in place on `state`.

    feedforward -> loss gradient / batch size -> backpropagate (all gradients from the
    weights as they were before this step) -> optimize (momentum on values and biases).
    `relu_masks[l]`, if given, replaces [A_l > 0] in the backward pass of hidden layer l
    (used when a pre-activation is within rounding of zero and two correct
    implementations may land on different sides).  Returns every intermediate.
    """
    L = len(state)
    X = np.ascontiguousarray(X, dtype=dtype)
    A, SA = mlp_forward(state, X, dtype, want_S=True)
    loss, S_loss, dZ_L, SdZ_L = softmax_ce(A[-1], labels, dtype)
    dZ = [None] * L; dA = [None] * L; SdA = [None] * L
    g = [None] * L; Sg = [None] * L; db = [None] * L; Sdb = [None] * L
    dZ[L - 1] = dZ_L
    for l in range(L - 1, -1, -1):
        st = state[l]
        if l < L - 1:
            if relu_masks is not None and relu_masks[l] is not None:
                dZ[l] = np.where(relu_masks[l], dA[l], 0).astype(dtype)
            else:
                dZ[l] = relu_backward(dA[l], A[l], dtype)
        inp = X if l == 0 else A[l - 1]
        g[l], Sg[l], db[l], Sdb[l] = sddmm(st["rows"], st["cols"], st["indptr"], st["indices"],
                                           dZ[l], inp, dtype)
        if l > 0:
            dA[l - 1], SdA[l - 1] = spmm_t(st["rows"], st["cols"], st["indptr"], st["indices"],
                                           st["values"], dZ[l], dtype)
    out = dict(A=A, SA=SA, loss=loss, S_loss=S_loss, dZ=dZ, SdZ_L=SdZ_L, dA=dA, SdA=SdA,
               g=g, Sg=Sg, db=db, Sdb=Sdb)
    if update:
        Sw, Sv, Sbw, Sbv = [], [], [], []
        for l, st in enumerate(state):
            st["values"], st["vel_w"], sw, sv = momentum(st["values"], st["vel_w"], g[l], lr, mu, Sg[l], dtype, nesterov)
            st["bias"], st["vel_b"], sbw, sbv = momentum(st["bias"], st["vel_b"], db[l], lr, mu, Sdb[l], dtype, nesterov)
            Sw.append(sw); Sv.append(sv); Sbw.append(sbw); Sbv.append(sbv)
        out.update(Sw=Sw, Sv=Sv, Sbw=Sbw, Sbv=Sbv)
    return out
