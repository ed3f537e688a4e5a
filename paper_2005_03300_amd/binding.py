"""ctypes marshalling for include/gcn.h.  No arithmetic happens here."""
from __future__ import annotations

import ctypes as C
import os
import re

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libgcn_hip.so")
_HEADER = os.path.join(os.path.dirname(HERE), "include", "gcn.h")

SYMMETRISE, ADD_SELF_LOOPS, NORM_SYM, BUILD_TRANSPOSE, NORM_ROW = 1, 2, 4, 8, 16
EPI_NONE, EPI_RELU, EPI_MASK = 0, 1, 2
ORDER_AUTO, ORDER_GEMM_FIRST, ORDER_SPMM_FIRST = 0, 1, 2
ACT_NONE, ACT_RELU = 0, 1
CFG_SPMM_ALGO, CFG_TIMING, CFG_SPMM_BLOCKS, CFG_SWEEP_HEAVY, CFG_SWEEP_WAVES, CFG_PATTERN_SPMM, CFG_HUB_MB, CFG_HUB_DMIN, CFG_HUB_BLOCK_COLS, CFG_SPLIT_LDS_KB, CFG_FUSED_LAST_LAYER = 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11

_lib = None


class GcnError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"gcn error {code}: {message}")
        self.code = code


def library_path() -> str:
    return _LIB_PATH


def exported_symbols():
    """Names of the functions include/gcn.h declares."""
    with open(_HEADER) as fh:
        text = fh.read()
    return sorted(set(re.findall(r"\b(gcn_[a-z_0-9]+)\s*\(", text)))


def lib():
    """Load libgcn_hip.so (torch first, so both share one HIP runtime)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2005_03300_amd.build` "
                "(there is no CPU fallback)")
        import torch  # noqa: F401  -- loads the HIP runtime the library binds to
        L = C.CDLL(_LIB_PATH)
        L.gcn_last_error.restype = C.c_char_p
        L.gcn_version.restype = C.c_char_p
        L.gcn_epoch_workspace_bytes.restype = C.c_size_t
        L.gcn_build_count.restype = C.c_int64
        _lib = L
    return _lib


def _check(rc: int):
    if rc != 0:
        raise GcnError(rc, lib().gcn_last_error().decode())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _ld(t) -> int:
    assert t.dim() == 2 and (t.shape[1] == 1 or t.stride(1) == 1), "rows must be contiguous"
    return t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


def _dev(t, dtype=None):
    import torch
    assert t.is_cuda, "device tensor expected"
    if dtype is not None:
        assert t.dtype == dtype, (t.dtype, dtype)
    return t


class Csr:
    """Owner of a gcn_csr handle."""

    def __init__(self, handle: int):
        self._h = C.c_void_p(handle)
        n, nnz, md = C.c_int64(), C.c_int64(), C.c_int32()
        _check(lib().gcn_csr_info(self._h, C.byref(n), C.byref(nnz), C.byref(md)))
        self.n, self.nnz, self.max_degree = n.value, nnz.value, md.value
        nr, nc = C.c_int64(), C.c_int64()
        _check(lib().gcn_csr_shape(self._h, C.byref(nr), C.byref(nc)))
        self.n_rows, self.n_cols = nr.value, nc.value

    def arrays(self, transposed: bool = False):
        """Copies of (rowptr, colidx, val, deg) as torch tensors on the device."""
        import torch
        rowptr = torch.empty((self.n_cols if transposed else self.n_rows) + 1, dtype=torch.int64, device="cuda")
        colidx = torch.empty(self.nnz, dtype=torch.int32, device="cuda")
        val = torch.empty(self.nnz, dtype=torch.float32, device="cuda")
        deg = torch.empty(self.n, dtype=torch.int32, device="cuda")
        _check(lib().gcn_csr_export(self._h, int(transposed), _ptr(rowptr), _ptr(colidx), _ptr(val), _ptr(deg),
                                    _stream()))
        return rowptr, colidx, val, deg

    def views(self, transposed: bool = False):
        """(rowptr, colidx, val, deg) as torch tensors that ALIAS the library's own device arrays (no copy):
        read-only for the caller, valid until close()."""
        import torch
        rp, ci, va, dg = C.c_void_p(), C.c_void_p(), C.c_void_p(), C.c_void_p()
        _check(lib().gcn_csr_arrays(self._h, int(transposed), C.byref(rp), C.byref(ci), C.byref(va), C.byref(dg)))

        class _Borrowed:
            def __init__(self, ptr, count, typestr):
                self.__cuda_array_interface__ = {"shape": (count,), "typestr": typestr, "data": (ptr, False),
                                                 "version": 2, "strides": None}

        def wrap(p, count, typestr, dtype):
            if count == 0 or not p.value:
                return torch.empty(0, dtype=dtype, device="cuda")
            return torch.as_tensor(_Borrowed(p.value, count, typestr), device="cuda")
        rows = self.n_cols if transposed else self.n_rows
        return (wrap(rp, rows + 1, "<i8", torch.int64), wrap(ci, self.nnz, "<i4", torch.int32),
                wrap(va, self.nnz, "<f4", torch.float32), wrap(dg, self.n, "<i4", torch.int32))

    def close(self):
        if self._h is not None and self._h.value:
            lib().gcn_csr_destroy(self._h)
        self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def gcn_csr_create(n: int, src, dst, flags: int) -> Csr:
    import torch
    src, dst = _dev(src, torch.int32).contiguous(), _dev(dst, torch.int32).contiguous()
    assert src.shape == dst.shape and src.dim() == 1
    out = C.c_void_p()
    _check(lib().gcn_csr_create(C.byref(out), C.c_int64(n), C.c_int64(src.shape[0]), _ptr(src), _ptr(dst),
                                C.c_uint32(flags), _stream()))
    return Csr(out.value)


def gcn_csr_create_from_csr(n: int, rowptr, colidx, val, flags: int) -> Csr:
    import torch
    rowptr = _dev(rowptr, torch.int64).contiguous()
    colidx = _dev(colidx, torch.int32).contiguous()
    if val is not None:
        val = _dev(val, torch.float32).contiguous()
    out = C.c_void_p()
    _check(lib().gcn_csr_create_from_csr(C.byref(out), C.c_int64(n), _ptr(rowptr), _ptr(colidx), _ptr(val),
                                         C.c_uint32(flags), _stream()))
    return Csr(out.value)


def gcn_csr_create_from_csr_rect(n_rows: int, n_cols: int, rowptr, colidx, val, flags: int) -> Csr:
    import torch
    rowptr = _dev(rowptr, torch.int64).contiguous()
    colidx = _dev(colidx, torch.int32).contiguous()
    if val is not None:
        val = _dev(val, torch.float32).contiguous()
    out = C.c_void_p()
    _check(lib().gcn_csr_create_from_csr_rect(C.byref(out), C.c_int64(n_rows), C.c_int64(n_cols), _ptr(rowptr),
                                              _ptr(colidx), _ptr(val), C.c_uint32(flags), _stream()))
    return Csr(out.value)


def gcn_spmm(a: Csr, trans: int, X, Z, epilogue: int = EPI_NONE, Zprev=None):
    import torch
    _dev(X, torch.float32), _dev(Z, torch.float32)
    f = X.shape[1]
    xr, zr = (a.n_rows, a.n_cols) if trans else (a.n_cols, a.n_rows)
    assert X.shape[0] == xr and tuple(Z.shape) == (zr, f)
    _check(lib().gcn_spmm(a._h, int(trans), C.c_int32(f), _ptr(X), C.c_int64(_ld(X)), _ptr(Z), C.c_int64(_ld(Z)),
                          int(epilogue), _ptr(Zprev), C.c_int64(_ld(Zprev) if Zprev is not None else 0), _stream()))
    return Z


def gcn_spmm_static(a: Csr, trans: int, X, Z, epilogue: int = EPI_NONE, Zprev=None):
    import torch
    _dev(X, torch.float32), _dev(Z, torch.float32)
    f = X.shape[1]
    xr, zr = (a.n_rows, a.n_cols) if trans else (a.n_cols, a.n_rows)
    assert X.shape[0] == xr and tuple(Z.shape) == (zr, f)
    _check(lib().gcn_spmm_static(a._h, int(trans), C.c_int32(f), _ptr(X), C.c_int64(_ld(X)), _ptr(Z),
                                 C.c_int64(_ld(Z)), int(epilogue), _ptr(Zprev),
                                 C.c_int64(_ld(Zprev) if Zprev is not None else 0), _stream()))
    return Z


def gcn_spmm_pattern(a: Csr, trans: int, X, Z, row_scale=None, epilogue: int = EPI_NONE, Zprev=None):
    import torch
    _dev(X, torch.float32), _dev(Z, torch.float32)
    f = X.shape[1]
    xr, zr = (a.n_rows, a.n_cols) if trans else (a.n_cols, a.n_rows)
    assert X.shape[0] == xr and tuple(Z.shape) == (zr, f)
    if row_scale is not None:
        _dev(row_scale, torch.float32)
        assert row_scale.numel() == zr and row_scale.is_contiguous()
    _check(lib().gcn_spmm_pattern(a._h, int(trans), C.c_int32(f), _ptr(X), C.c_int64(_ld(X)), _ptr(Z),
                                  C.c_int64(_ld(Z)), _ptr(row_scale), int(epilogue), _ptr(Zprev),
                                  C.c_int64(_ld(Zprev) if Zprev is not None else 0), _stream()))
    return Z


def gcn_scale_rows(X, scale, Y):
    import torch
    _dev(X, torch.float32), _dev(scale, torch.float32), _dev(Y, torch.float32)
    rows, cols = X.shape
    assert tuple(Y.shape) == (rows, cols) and scale.numel() == rows and scale.is_contiguous()
    _check(lib().gcn_scale_rows(C.c_int64(rows), C.c_int32(cols), _ptr(X), C.c_int64(_ld(X)), _ptr(scale), _ptr(Y),
                                C.c_int64(_ld(Y)), _stream()))
    return Y


def gcn_csr_inv_sqrt_degrees(a: Csr, out):
    import torch
    _dev(out, torch.float32)
    assert out.numel() == a.n_rows and out.is_contiguous()
    _check(lib().gcn_csr_inv_sqrt_degrees(a._h, _ptr(out), _stream()))
    return out


def gcn_gemm(ta: int, tb: int, A, B, Cm, bias=None, epilogue: int = EPI_NONE, Zprev=None):
    import torch
    _dev(A, torch.float32), _dev(B, torch.float32), _dev(Cm, torch.float32)
    M, N = Cm.shape
    K = A.shape[0] if ta else A.shape[1]
    _check(lib().gcn_gemm(int(ta), int(tb), C.c_int64(M), C.c_int64(N), C.c_int64(K), _ptr(A), C.c_int64(_ld(A)),
                          _ptr(B), C.c_int64(_ld(B)), _ptr(Cm), C.c_int64(_ld(Cm)), _ptr(bias), int(epilogue),
                          _ptr(Zprev), C.c_int64(_ld(Zprev) if Zprev is not None else 0), _stream()))
    return Cm


def gcn_relu(Z, H):
    _check(lib().gcn_relu(C.c_int64(Z.shape[0]), C.c_int32(Z.shape[1]), _ptr(Z), C.c_int64(_ld(Z)), _ptr(H),
                          C.c_int64(_ld(H)), _stream()))
    return H


def gcn_relu_mask(G, Zprev, out):
    _check(lib().gcn_relu_mask(C.c_int64(G.shape[0]), C.c_int32(G.shape[1]), _ptr(G), C.c_int64(_ld(G)), _ptr(Zprev),
                               C.c_int64(_ld(Zprev)), _ptr(out), C.c_int64(_ld(out)), _stream()))
    return out


def gcn_softmax_nll(Z, labels, loss, G=None):
    import torch
    _dev(Z, torch.float32), _dev(labels, torch.int32), _dev(loss, torch.float32)
    _check(lib().gcn_softmax_nll(C.c_int64(Z.shape[0]), C.c_int32(Z.shape[1]), _ptr(Z), C.c_int64(_ld(Z)),
                                 _ptr(labels), _ptr(loss), _ptr(G), C.c_int64(_ld(G) if G is not None else 0),
                                 _stream()))
    return loss


def gcn_softmax_nll_masked(Z, labels, n_labelled: int, loss, G=None):
    import torch
    _dev(Z, torch.float32), _dev(labels, torch.int32), _dev(loss, torch.float32)
    _check(lib().gcn_softmax_nll_masked(C.c_int64(Z.shape[0]), C.c_int32(Z.shape[1]), _ptr(Z), C.c_int64(_ld(Z)),
                                        _ptr(labels), C.c_int64(n_labelled), _ptr(loss), _ptr(G),
                                        C.c_int64(_ld(G) if G is not None else 0), _stream()))
    return loss


def gcn_layer_forward(a: Csr, Hin, W, Z, Hout, T, order: int = ORDER_AUTO, act: int = ACT_RELU, bias=None):
    f_in, f_out = W.shape
    assert W.is_contiguous() and Z.is_contiguous() and T.is_contiguous()
    assert Hout is None or Hout.is_contiguous()
    _check(lib().gcn_layer_forward(a._h, C.c_int32(f_in), C.c_int32(f_out), _ptr(Hin), C.c_int64(_ld(Hin)), _ptr(W),
                                   _ptr(bias), _ptr(Z), _ptr(Hout), _ptr(T), int(order), int(act), _stream()))


def gcn_layer_backward(a: Csr, Hin, Zprev, W, G, T, S, Y, Gprev, order: int = ORDER_AUTO, dbias=None):
    f_in, f_out = W.shape
    for t in (W, G, S, Y):
        assert t.is_contiguous()
    _check(lib().gcn_layer_backward(a._h, C.c_int32(f_in), C.c_int32(f_out), _ptr(Hin),
                                    C.c_int64(_ld(Hin) if Hin is not None else 0), _ptr(Zprev), _ptr(W), _ptr(G),
                                    _ptr(T), _ptr(S), _ptr(Y), _ptr(dbias), _ptr(Gprev), int(order), _stream()))


def _dims_array(dims):
    return (C.c_int32 * len(dims))(*[int(d) for d in dims])


def gcn_epoch_workspace_bytes(n: int, dims, order: int = ORDER_AUTO) -> int:
    return int(lib().gcn_epoch_workspace_bytes(C.c_int64(n), C.c_int32(len(dims) - 1), _dims_array(dims), int(order)))


def gcn_epoch(a: Csr, dims, H0, labels, W, Y, lr: float, loss, workspace, order: int = ORDER_AUTO):
    L = len(dims) - 1
    assert len(W) == L and len(Y) == L and H0.is_contiguous()
    Wp = (C.c_void_p * L)(*[w.data_ptr() for w in W])
    Yp = (C.c_void_p * L)(*[y.data_ptr() for y in Y])
    _check(lib().gcn_epoch(a._h, C.c_int32(L), _dims_array(dims), _ptr(H0), _ptr(labels), Wp, Yp, C.c_float(lr),
                           _ptr(loss), _ptr(workspace), C.c_size_t(workspace.numel() * workspace.element_size()),
                           int(order), _stream()))
    return loss


def gcn_epoch_masked(a: Csr, dims, H0, labels, n_labelled: int, W, Y, lr: float, loss, workspace,
                     order: int = ORDER_AUTO):
    L = len(dims) - 1
    assert len(W) == L and len(Y) == L and H0.is_contiguous()
    Wp = (C.c_void_p * L)(*[w.data_ptr() for w in W])
    Yp = (C.c_void_p * L)(*[y.data_ptr() for y in Y])
    _check(lib().gcn_epoch_masked(a._h, C.c_int32(L), _dims_array(dims), _ptr(H0), _ptr(labels),
                                  C.c_int64(n_labelled), Wp, Yp, C.c_float(lr), _ptr(loss), _ptr(workspace),
                                  C.c_size_t(workspace.numel() * workspace.element_size()), int(order), _stream()))
    return loss


def gcn_epoch_preaggregated(a: Csr, dims, P0, labels, n_labelled: int, W, Y, lr: float, loss, workspace,
                            order: int = ORDER_AUTO):
    L = len(dims) - 1
    assert len(W) == L and len(Y) == L and P0.is_contiguous() and tuple(P0.shape) == (a.n, dims[0])
    Wp = (C.c_void_p * L)(*[w.data_ptr() for w in W])
    Yp = (C.c_void_p * L)(*[y.data_ptr() for y in Y])
    _check(lib().gcn_epoch_preaggregated(a._h, C.c_int32(L), _dims_array(dims), _ptr(P0), _ptr(labels),
                                         C.c_int64(n_labelled), Wp, Yp, C.c_float(lr), _ptr(loss), _ptr(workspace),
                                         C.c_size_t(workspace.numel() * workspace.element_size()), int(order),
                                         _stream()))
    return loss


def gcn_epoch_view(n: int, dims, order: int, workspace, layer: int):
    """(Z^l, G^l) of the last gcn_epoch call as torch tensors aliasing the workspace."""
    import torch
    Zp, Gp = C.c_void_p(), C.c_void_p()
    _check(lib().gcn_epoch_view(C.c_int64(n), C.c_int32(len(dims) - 1), _dims_array(dims), int(order), _ptr(workspace),
                                C.c_int32(layer), C.byref(Zp), C.byref(Gp)))
    base = workspace.data_ptr()
    flat = workspace.view(torch.uint8).view(-1)
    f = int(dims[layer])

    def view(p):
        off = p.value - base
        return flat[off:off + n * f * 4].view(torch.float32).view(n, f)
    return view(Zp), view(Gp)


def gcn_config(key: int, value: int):
    _check(lib().gcn_config(int(key), int(value)))


def gcn_csr_config(a: Csr, key: int, value: int):
    _check(lib().gcn_csr_config(a._h, int(key), int(value)))


def gcn_spmm_prepare(a: Csr, trans: int, f: int):
    _check(lib().gcn_spmm_prepare(a._h, int(trans), C.c_int32(f), _stream()))


def gcn_spmm_describe(a: Csr, trans: int, f: int) -> str:
    buf = C.create_string_buffer(1024)
    _check(lib().gcn_spmm_describe(a._h, int(trans), C.c_int32(f), buf, C.c_size_t(1024), _stream()))
    return buf.value.decode()


def gcn_epoch_prepare(a: Csr, dims, order: int = ORDER_AUTO):
    _check(lib().gcn_epoch_prepare(a._h, C.c_int32(len(dims) - 1), _dims_array(dims), int(order), _stream()))


def gcn_scratch_release():
    _check(lib().gcn_scratch_release())


def gcn_build_count() -> int:
    return int(lib().gcn_build_count())


def gcn_csr_last_spmm_schedule(a: Csr) -> int:
    return int(lib().gcn_csr_last_spmm_schedule(a._h))


def gcn_timing_read():
    cnt, ms = C.c_int64(), C.c_double()
    _check(lib().gcn_timing_read(C.byref(cnt), C.byref(ms)))
    return cnt.value, ms.value


def gcn_timing_read_phases():
    """Returns {phase name: (spans, total ms)} and resets the record."""
    cnt = (C.c_int64 * 4)()
    ms = (C.c_double * 4)()
    _check(lib().gcn_timing_read_phases(cnt, ms))
    names = ("spmm_kernel", "spmm", "gemm", "other")
    return {k: (cnt[i], ms[i]) for i, k in enumerate(names)}


def gcn_radix_sort(keys, payload=None, end_bit=None, descending=False):
    """Stable radix sort of a 1-D tensor of 4- or 8-byte keys (their bit patterns as unsigned); payload: [n, w]
    int32 tensor with w in 1..3, or None.  Returns (sorted_keys, moved_payload or None)."""
    import torch
    keys = _dev(keys).contiguous()
    kb = keys.element_size()
    n = keys.numel()
    out = torch.empty_like(keys)
    pb, pout = 0, None
    if payload is not None:
        payload = _dev(payload, torch.int32).contiguous()
        assert payload.dim() == 2 and payload.shape[0] == n
        pb = 4 * payload.shape[1]
        pout = torch.empty_like(payload)
    _check(lib().gcn_radix_sort(C.c_int64(n), kb, _ptr(keys), _ptr(out), pb, _ptr(payload), _ptr(pout),
                                8 * kb if end_bit is None else int(end_bit), int(bool(descending)), _stream()))
    return out, pout


def gcn_exclusive_scan_i64(x, out=None):
    import torch
    x = _dev(x, torch.int64).contiguous()
    out = torch.empty_like(x) if out is None else _dev(out, torch.int64)
    _check(lib().gcn_exclusive_scan_i64(C.c_int64(x.numel()), _ptr(x), _ptr(out), _stream()))
    return out


def gcn_unique_u64(keys):
    """First key of every run of equal neighbours of an int64 tensor (bit patterns); returns the kept prefix."""
    import torch
    keys = _dev(keys, torch.int64).contiguous()
    out = torch.empty_like(keys)
    cnt = C.c_int64(0)
    _check(lib().gcn_unique_u64(C.c_int64(keys.numel()), _ptr(keys), _ptr(out), C.byref(cnt), _stream()))
    return out[:cnt.value]


def gcn_last_spmm_schedule() -> int:
    return int(lib().gcn_last_spmm_schedule())


SCHED_ROWWISE, SCHED_SPLIT, SCHED_SWEEP, SCHED_HUB, SCHED_BLOCKED = 1, 2, 3, 4, 5


def gcn_version() -> str:
    return lib().gcn_version().decode()
