"""CPU ORACLE -- TEST INFRASTRUCTURE ONLY.

Plain, slow reference for the GCN hot path, written from the paper's definitions (sections
"Graph Neural Networks", "Forward Propagation", "Backpropagation Derivations").  Only tests,
the smoke check and the benchmark's cpu_baseline leg may import this package; the GPU library
and its Python binding never do, and this package never imports them.

The loops live in ``gcn_oracle.c`` (compiled for float and for double storage); this module
marshals numpy arrays and composes the per-layer and per-epoch formulas in the paper's order.
Dense arrays of dtype float32 use the float build, float64 the double build; sums are always
accumulated in double.

Readings of the paper taken here (each is listed with its reason in the design notes):
  * Equation 1's prose has sigma and Z swapped; H = sigma(Z) as in "Forward Propagation".
  * Equation 3 labels the gradient Y^{l-1}; it is the gradient of the weight that produces
    Z^l, i.e. dL/dW^l = (H^{l-1})^T A G^l (confirmed by finite differences in the tests).
  * The last layer's activation is a row-wise log-softmax; the loss is the mean negative
    log-likelihood over all vertices, which makes G^L = (softmax(Z^L) - onehot(y)) / n.
  * sigma'(z) = 1 for z > 0 and 0 otherwise.
  * Input self-loops are dropped and duplicates collapse; exactly one diagonal entry is added.

Parity pins: every function here is pinned by tests/test_oracle_pins.py (brute force on tiny
inputs in pure Python, closed forms, invariants, finite differences).  No function is
"parity unpinned".
"""
from __future__ import annotations

import ctypes as C
import dataclasses

import numpy as np

from . import build as _build

_libs: dict = {}

_i64p = C.POINTER(C.c_int64)
_i32p = C.POINTER(C.c_int32)
_u64p = C.POINTER(C.c_uint64)
_f32p = C.POINTER(C.c_float)


def _lib(kind: str):
    if kind not in _libs:
        _build.build(force=False)
        lib = C.CDLL(_build.LIBS[kind][1])
        lib.orc_edge_set.restype = C.c_int64
        lib.orc_softmax_nll.restype = C.c_double
        _libs[kind] = lib
    return _libs[kind]


def _kind(a: np.ndarray) -> str:
    if a.dtype == np.float32:
        return "f32"
    if a.dtype == np.float64:
        return "f64"
    raise TypeError(f"dense arrays must be float32 or float64, got {a.dtype}")


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _ld(X: np.ndarray) -> int:
    """Leading dimension (in elements) of a 2-D array whose rows are contiguous."""
    assert X.ndim == 2 and (X.shape[1] == 1 or X.strides[1] == X.itemsize)
    assert X.strides[0] % X.itemsize == 0 and X.strides[0] >= X.shape[1] * X.itemsize
    return X.strides[0] // X.itemsize


def threads() -> int:
    return int(_lib("f32").orc_threads())


def set_threads(count: int) -> None:
    """Threads used by the loops from now on (for timing on one core); results do not depend on it."""
    for kind in ("f32", "f64"):
        _lib(kind).orc_set_threads(int(count))


# ---------------------------------------------------------------------------------------------
# graph
# ---------------------------------------------------------------------------------------------

@dataclasses.dataclass
class Csr:
    """Compressed rows: rowptr int64 [n+1], colidx int32 [nnz] ascending per row, val float32
    [nnz], deg int32 [n] = stored entries per row of the UNtransposed matrix."""
    n: int
    rowptr: np.ndarray
    colidx: np.ndarray
    val: np.ndarray
    deg: np.ndarray
    ncols: int = -1          # -1: square

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    @property
    def n_cols(self) -> int:
        return self.n if self.ncols < 0 else self.ncols


def build_csr(n, src, dst, symmetrise=True, self_loops=True, norm="sym", transpose=False) -> Csr:
    """Modified adjacency matrix of section "Graph Neural Networks" from a raw edge list.

    ``transpose=True`` returns the transposed matrix, built on its own by sorting the same
    entry set by (column, row) rather than by transposing the first result.  ``norm`` is
    "sym" (entries 1/sqrt(d_i d_j), d = row degrees of the untransposed matrix), "row" (entries
    1/d_i, the row normalisation used for directed graphs) or "none" (entries 1)."""
    lib = _lib("f32")
    src = np.ascontiguousarray(src, np.int32)
    dst = np.ascontiguousarray(dst, np.int32)
    m = src.shape[0]
    keys = np.empty(2 * m + n, np.uint64)
    cnt = lib.orc_edge_set(C.c_int64(n), C.c_int64(m), _p(src), _p(dst), int(symmetrise),
                           int(self_loops), 0, _p(keys))
    if cnt < 0:
        raise ValueError("vertex id outside [0, n)")
    rowptr = np.empty(n + 1, np.int64)
    colidx = np.empty(cnt, np.int32)
    lib.orc_compress(C.c_int64(n), C.c_int64(cnt), _p(keys), _p(rowptr), _p(colidx))
    deg = np.empty(n, np.int32)
    lib.orc_degrees(C.c_int64(n), _p(rowptr), _p(deg))
    if transpose:
        cnt_t = lib.orc_edge_set(C.c_int64(n), C.c_int64(m), _p(src), _p(dst), int(symmetrise),
                                 int(self_loops), 1, _p(keys))
        assert cnt_t == cnt
        rowptr = np.empty(n + 1, np.int64)
        colidx = np.empty(cnt, np.int32)
        lib.orc_compress(C.c_int64(n), C.c_int64(cnt), _p(keys), _p(rowptr), _p(colidx))
    del keys
    val = np.empty(cnt, np.float32)
    if norm == "sym":
        lib.orc_values_sym(C.c_int64(n), _p(rowptr), _p(colidx), _p(deg), _p(val))
    elif norm == "row":
        lib.orc_values_row(C.c_int64(n), _p(rowptr), _p(colidx), _p(deg), int(transpose), _p(val))
    elif norm == "none":
        val[:] = 1.0
    else:
        raise ValueError(norm)
    return Csr(n, rowptr, colidx, val, deg)


def slice_rows(A: Csr, r0: int, r1: int) -> Csr:
    """Rows [r0, r1) of A as an (r1-r0) x n_cols matrix: one process's block row in the paper's 1D
    algorithm ("A One-Dimensional (1D) Algorithm")."""
    lo, hi = int(A.rowptr[r0]), int(A.rowptr[r1])
    return Csr(r1 - r0, (A.rowptr[r0:r1 + 1] - lo).astype(np.int64), A.colidx[lo:hi].copy(), A.val[lo:hi].copy(),
               A.deg[r0:r1].copy(), A.n_cols)


def transpose(A: Csr) -> Csr:
    """A^T in compressed rows, by the definition: entry (i,j,v) becomes (j,i,v); rows of the result
    ascend in i because the stable sort keeps the row-major input order."""
    rows = np.repeat(np.arange(A.n, dtype=np.int64), np.diff(A.rowptr))
    order = np.argsort(A.colidx, kind="stable")
    counts = np.bincount(A.colidx, minlength=A.n_cols)
    rowptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    return Csr(A.n_cols, rowptr, rows[order].astype(np.int32), A.val[order].copy(), A.deg, A.n)


# ---------------------------------------------------------------------------------------------
# primitives
# ---------------------------------------------------------------------------------------------

def spmm(A: Csr, X: np.ndarray) -> np.ndarray:
    """Z = A X with Z[i,:] = sum over stored entries k of row i of val[k] X[col[k],:]."""
    assert X.shape[0] == A.n_cols
    k = _kind(X)
    f = X.shape[1]
    Z = np.empty((A.n, f), X.dtype)
    _lib(k).orc_spmm(C.c_int64(A.n), _p(A.rowptr), _p(A.colidx), _p(A.val), C.c_int32(f),
                     _p(X), C.c_int64(_ld(X)), _p(Z), C.c_int64(f))
    return Z


def spmm_rows(A: Csr, X: np.ndarray, rows) -> np.ndarray:
    """Rows ``rows`` of A X, one at a time (for spot checks at sizes too big for a full product)."""
    assert X.shape[0] == A.n_cols
    k = _kind(X)
    rows = np.ascontiguousarray(rows, np.int64)
    f = X.shape[1]
    Z = np.empty((rows.shape[0], f), X.dtype)
    _lib(k).orc_spmm_rows(C.c_int64(rows.shape[0]), _p(rows), _p(A.rowptr), _p(A.colidx), _p(A.val),
                          C.c_int32(f), _p(X), C.c_int64(_ld(X)), _p(Z))
    return Z


def inv_sqrt_degrees(A: Csr) -> np.ndarray:
    """s_i = (float)(1/sqrt(d_i)) with d the stored entries per row of the untransposed matrix."""
    s = np.empty(A.deg.shape[0], np.float32)
    _lib("f32").orc_inv_sqrt_deg(C.c_int64(s.shape[0]), _p(A.deg), _p(s))
    return s


def scale_rows(X: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """Y[i,:] = scale[i] X[i,:], rounded once to the type of X."""
    k = _kind(X)
    scale = np.ascontiguousarray(scale, np.float32)
    assert scale.shape[0] == X.shape[0]
    Y = np.empty(X.shape, X.dtype)
    _lib(k).orc_scale_rows(C.c_int64(X.shape[0]), C.c_int32(X.shape[1]), _p(X), C.c_int64(_ld(X)), _p(scale),
                           _p(Y), C.c_int64(X.shape[1]))
    return Y


def spmm_pattern(A: Csr, X: np.ndarray, row_scale=None) -> np.ndarray:
    """Z[i,:] = row_scale[i] * sum over stored entries k of row i of X[col[k],:] (stored values ignored)."""
    assert X.shape[0] == A.n_cols
    k = _kind(X)
    f = X.shape[1]
    Z = np.empty((A.n, f), X.dtype)
    if row_scale is not None:
        row_scale = np.ascontiguousarray(row_scale, np.float32)
        assert row_scale.shape[0] == A.n
    _lib(k).orc_spmm_pattern(C.c_int64(A.n), _p(A.rowptr), _p(A.colidx), _p(row_scale) if row_scale is not None else None,
                             C.c_int32(f), _p(X), C.c_int64(_ld(X)), _p(Z), C.c_int64(f))
    return Z


def gemm(A: np.ndarray, B: np.ndarray, ta: bool = False, tb: bool = False) -> np.ndarray:
    """op(A) op(B) by the textbook triple loop."""
    A = np.ascontiguousarray(A)
    B = np.ascontiguousarray(B)
    assert A.dtype == B.dtype
    k = _kind(A)
    M, K = (A.shape[1], A.shape[0]) if ta else A.shape
    K2, N = (B.shape[1], B.shape[0]) if tb else B.shape
    assert K == K2, (A.shape, B.shape, ta, tb)
    Cm = np.empty((M, N), A.dtype)
    _lib(k).orc_gemm(int(ta), int(tb), C.c_int64(M), C.c_int64(N), C.c_int64(K), _p(A),
                     C.c_int64(A.shape[1]), _p(B), C.c_int64(B.shape[1]), _p(Cm), C.c_int64(N))
    return Cm


def relu(Z: np.ndarray) -> np.ndarray:
    Z = np.ascontiguousarray(Z)
    H = np.empty_like(Z)
    _lib(_kind(Z)).orc_relu(C.c_int64(Z.size), _p(Z), _p(H))
    return H


def relu_mask(G: np.ndarray, Z: np.ndarray) -> np.ndarray:
    """G (Hadamard) sigma'(Z)."""
    G = np.ascontiguousarray(G)
    Z = np.ascontiguousarray(Z)
    assert G.shape == Z.shape and G.dtype == Z.dtype
    out = np.empty_like(G)
    _lib(_kind(G)).orc_relu_mask(C.c_int64(G.size), _p(G), _p(Z), _p(out))
    return out


def softmax_nll(Z: np.ndarray, labels: np.ndarray, want_grad: bool = True):
    """Mean NLL of row-wise log-softmax(Z) over the vertices with label >= 0 (negative labels mark
    vertices outside the training split) and its gradient with respect to Z (Equation 1)."""
    Z = np.ascontiguousarray(Z)
    labels = np.ascontiguousarray(labels, np.int32)
    n, Cn = Z.shape
    assert labels.shape == (n,) and labels.max() < Cn
    G = np.empty_like(Z) if want_grad else None
    loss = _lib(_kind(Z)).orc_softmax_nll(C.c_int64(n), C.c_int32(Cn), _p(Z), C.c_int64(Cn), _p(labels),
                                          _p(G) if want_grad else None, C.c_int64(Cn))
    return float(loss), G


def sgd(W: np.ndarray, Y: np.ndarray, lr: float) -> np.ndarray:
    W = np.array(W, copy=True, order="C")
    Y = np.ascontiguousarray(Y)
    _lib(_kind(W)).orc_sgd(C.c_int64(W.size), _p(W), _p(Y), C.c_double(lr))
    return W


# ---------------------------------------------------------------------------------------------
# layers and the epoch, in the paper's order
# ---------------------------------------------------------------------------------------------

def layer_forward(At: Csr, Hin: np.ndarray, W: np.ndarray, act: str = "relu", bias=None):
    """"Forward Propagation": Z = A^T (Hin W), H = sigma(Z).  ``At`` holds A^T in compressed
    rows.  ``act`` is "relu" or "none" (the last layer's log-softmax lives in softmax_nll).
    An optional bias row is added to every row of Z (the paper has none)."""
    Z = spmm(At, gemm(Hin, W))
    if bias is not None:
        Z = (Z.astype(np.float64) + np.asarray(bias, np.float64)[None, :]).astype(Z.dtype)
    H = relu(Z) if act == "relu" else Z.copy()
    return Z, H


def layer_backward(A: Csr, Hin: np.ndarray, Zprev, W: np.ndarray, G: np.ndarray):
    """Equations 2 and 3 for the layer whose weight is W and whose dL/dZ is G:
         S = A G                      (computed once, used twice)
         Y = Hin^T S                  (gradient of W)
         Gprev = (S W^T) (Hadamard) sigma'(Zprev)      (skipped when Zprev is None)
    Returns (S, Y, Gprev, dbias) with dbias = column sums of G."""
    S = spmm(A, G)
    Y = gemm(Hin, S, ta=True)
    Gprev = None
    if Zprev is not None:
        Gprev = relu_mask(gemm(S, W, tb=True), Zprev)
    dbias = G.astype(np.float64).sum(axis=0).astype(G.dtype)
    return S, Y, Gprev, dbias


def forward(At: Csr, H0: np.ndarray, Ws):
    """All layers; returns the lists Z[1..L] and H[0..L] (H[L] = Z[L], pre-softmax)."""
    Hs, Zs = [H0], []
    for l, W in enumerate(Ws):
        Z, H = layer_forward(At, Hs[-1], W, "relu" if l + 1 < len(Ws) else "none")
        Zs.append(Z)
        Hs.append(H)
    return Zs, Hs


def epoch(A: Csr, At: Csr, H0: np.ndarray, labels: np.ndarray, Ws, lr: float = 0.0, sign_from=None):
    """One full-batch epoch: forward, loss, backward (Equations 1-3) and, if lr != 0, the
    gradient step.  Returns dict(loss, Y=[...], W=[...], Z=[...], H=[...], G=[...]).

    ``sign_from`` (optional, one array per hidden layer, or None entries): sigma'(Z^l) of Equation 2
    is then taken from the sign of ``sign_from[l]`` instead of this function's own Z^l.  sigma' is a
    decision (z > 0 or not) that floating point takes; a caller that checks an fp32 implementation
    passes that implementation's own pre-activations (or its H = ReLU(Z), which has the same sign
    pattern) so that both sides take the decision on the same numbers, and checks separately that
    the two sign patterns differ only where Z^l is zero to rounding.  The forward pass and the loss
    never use it."""
    Zs, Hs = forward(At, H0, Ws)
    loss, G = softmax_nll(Zs[-1], labels)
    Ys = [None] * len(Ws)
    Gs = [None] * len(Ws)
    for l in range(len(Ws) - 1, -1, -1):
        Gs[l] = G
        Zprev = None
        if l > 0:
            Zprev = Zs[l - 1]
            if sign_from is not None and sign_from[l - 1] is not None:
                Zprev = np.ascontiguousarray(sign_from[l - 1]).astype(Zprev.dtype)
                assert Zprev.shape == Zs[l - 1].shape
        _, Ys[l], G, _ = layer_backward(A, Hs[l], Zprev, Ws[l], G)
    newW = [sgd(W, Y, lr) if lr != 0.0 else W for W, Y in zip(Ws, Ys)]
    return dict(loss=loss, Y=Ys, W=newW, Z=Zs, H=Hs, G=Gs)


def loss_only(At: Csr, H0: np.ndarray, labels: np.ndarray, Ws) -> float:
    Zs, _ = forward(At, H0, Ws)
    return softmax_nll(Zs[-1], labels, want_grad=False)[0]
