"""ctypes view of libasteria.so.  Functions carry the names of the C entry points; they take
torch tensors on the GPU, build the host descriptor arrays and pass raw pointers.  Nothing is
computed here, and there is no fallback: a missing library is an ImportError."""
from __future__ import annotations

import ctypes
import os
from ctypes import c_float, c_int, c_int32, c_size_t, c_void_p, POINTER, Structure
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libasteria.so")

OK, INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, HIP_ERROR, EXCEEDS_STATIC_SCRATCH = range(6)
F32, BF16 = 0, 1
ACC_F32, ACC_F64 = 0, 1
LAYOUT_FULL, LAYOUT_PACKED = 0, 1
EPS_RELATIVE, EPS_ABSOLUTE = 0, 1
INFO_OK, INFO_NOT_CONVERGED, INFO_NOT_PD = 0, 1, 2


class AsteriaError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__(f"{where}: {status_string(status)} (status {status})")
        self.status = status


class _Block(Structure):
    _fields_ = [("G", c_void_p), ("L", c_void_p), ("R", c_void_p), ("m", c_int32), ("n", c_int32),
                ("ldg", c_int32), ("ldl", c_int32), ("ldr", c_int32), ("g_dtype", c_int32), ("acc", c_int32), ("lr_layout", c_int32)]


class _Factor(Structure):
    _fields_ = [("A", c_void_p), ("X", c_void_p), ("n", c_int32), ("lda", c_int32), ("ldx", c_int32),
                ("a_layout", c_int32)]


class _SymPair(Structure):
    _fields_ = [("full", c_void_p), ("packed", c_void_p), ("n", c_int32), ("ld", c_int32)]


class _PBlock(Structure):
    _fields_ = [("XL", c_void_p), ("G", c_void_p), ("XR", c_void_p), ("P", c_void_p),
                ("m", c_int32), ("n", c_int32), ("ldxl", c_int32), ("ldg", c_int32),
                ("ldxr", c_int32), ("ldp", c_int32), ("g_dtype", c_int32), ("p_dtype", c_int32)]


class _SBlock(Structure):
    _fields_ = [("G", c_void_p), ("QL", c_void_p), ("QR", c_void_p), ("M", c_void_p), ("V", c_void_p),
                ("N", c_void_p), ("m", c_int32), ("n", c_int32), ("ldg", c_int32), ("ldql", c_int32),
                ("ldqr", c_int32), ("ldm", c_int32), ("ldv", c_int32), ("ldn", c_int32),
                ("g_dtype", c_int32), ("ldqlt", c_int32), ("ldqrt", c_int32), ("QLt", c_void_p), ("QRt", c_void_p)]


class _TPair(Structure):
    _fields_ = [("src", c_void_p), ("dst", c_void_p), ("rows", c_int32), ("cols", c_int32), ("lds", c_int32),
                ("ldd", c_int32)]


class _RBlock(Structure):
    _fields_ = [("QL_old", c_void_p), ("QL_new", c_void_p), ("QR_old", c_void_p), ("QR_new", c_void_p),
                ("M", c_void_p), ("V", c_void_p), ("permL", c_void_p), ("permR", c_void_p),
                ("m", c_int32), ("n", c_int32), ("ldql_old", c_int32), ("ldql_new", c_int32),
                ("ldqr_old", c_int32), ("ldqr_new", c_int32), ("ldm", c_int32), ("ldv", c_int32)]


class SoapRefreshOpts(Structure):
    """Mirror of asteria_soap_refresh_opts."""
    _fields_ = [("sort", c_int32), ("from_identity", c_int32), ("rounds", c_int32), ("n_aux", c_int32),
                ("aux_streams", POINTER(c_void_p)), ("Xt", POINTER(c_void_p)), ("ldxt", POINTER(c_int32)),
                ("xt_in", c_int32)]


class RootOpts(Structure):
    """Mirror of asteria_root_opts; constructed with the library defaults."""
    _fields_ = [("max_iters", c_int32), ("fp64_iters", c_int32), ("power_iters", c_int32),
                ("schedule", c_int32), ("stop_resid", c_float), ("power_tol", c_float),
                ("lambda_margin", c_float), ("lowp_from", c_int32), ("int8_slices", c_int32)]

    def __init__(self, **kw):
        super().__init__()
        lib().asteria_root_opts_default(ctypes.byref(self))
        for k, v in kw.items():
            if k not in dict(self._fields_):
                raise TypeError(f"unknown option {k}")
            setattr(self, k, v)


_lib = None


def library_path() -> str:
    return _LIB_PATH


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2605_16184_amd.build` "
                              "(there is no fallback path)")
        L = ctypes.CDLL(_LIB_PATH)
        L.asteria_version.restype = c_int
        L.asteria_status_string.restype = ctypes.c_char_p
        L.asteria_status_string.argtypes = [c_int]
        L.asteria_root_opts_default.argtypes = [POINTER(RootOpts)]
        L.asteria_root_opts_default.restype = None
        L.asteria_stats_update_workspace_bytes.restype = c_size_t
        L.asteria_stats_update_workspace_bytes.argtypes = [POINTER(_Block), c_int]
        L.asteria_stats_update.restype = c_int
        L.asteria_stats_update.argtypes = [POINTER(_Block), c_int, c_float, c_void_p, c_size_t, c_void_p]
        L.asteria_inverse_root_workspace_bytes.restype = c_size_t
        L.asteria_inverse_root_workspace_bytes.argtypes = [POINTER(_Factor), c_int, POINTER(RootOpts),
                                                           POINTER(c_size_t)]
        L.asteria_inverse_root_plan.restype = c_int
        L.asteria_inverse_root_plan.argtypes = [c_int, c_int, POINTER(c_float), c_int, POINTER(RootOpts),
                                                POINTER(c_int32), POINTER(c_int32), POINTER(c_int32)]
        L.asteria_inverse_root.restype = c_int
        L.asteria_inverse_root.argtypes = [POINTER(_Factor), c_int, c_int, c_int, POINTER(c_float), c_int,
                                           POINTER(RootOpts), c_void_p, c_void_p, c_void_p, c_void_p,
                                           c_void_p, c_size_t, c_void_p]
        L.asteria_static_scratch_bytes.restype = c_size_t
        L.asteria_static_scratch_bytes.argtypes = []
        L.asteria_inverse_root_static.restype = c_int
        L.asteria_inverse_root_static.argtypes = [POINTER(_Factor), c_int, c_int, c_int, POINTER(c_float), c_int,
                                                  POINTER(RootOpts), c_void_p, c_void_p, c_void_p, c_void_p,
                                                  c_void_p]
        L.asteria_precondition_workspace_bytes.restype = c_size_t
        L.asteria_precondition_workspace_bytes.argtypes = [POINTER(_PBlock), c_int]
        L.asteria_precondition.restype = c_int
        L.asteria_precondition.argtypes = [POINTER(_PBlock), c_int, c_void_p, c_size_t, c_void_p]
        L.asteria_soap_refresh_workspace_bytes.restype = c_size_t
        L.asteria_soap_refresh_workspace_bytes.argtypes = [POINTER(_Factor), c_int, POINTER(c_size_t)]
        L.asteria_soap_refresh.restype = c_int
        L.asteria_soap_refresh.argtypes = [POINTER(_Factor), c_int, c_void_p, c_void_p, c_size_t, c_void_p]
        L.asteria_soap_refresh_opts_default.restype = None
        L.asteria_soap_refresh_opts_default.argtypes = [POINTER(SoapRefreshOpts)]
        L.asteria_soap_refresh_ex.restype = c_int
        L.asteria_soap_refresh_ex.argtypes = [POINTER(_Factor), c_int, POINTER(SoapRefreshOpts), c_void_p, c_void_p,
                                              c_void_p, c_size_t, c_void_p]
        L.asteria_soap_reproject_workspace_bytes.restype = c_size_t
        L.asteria_soap_reproject_workspace_bytes.argtypes = [POINTER(_RBlock), c_int]
        L.asteria_soap_reproject.restype = c_int
        L.asteria_soap_reproject.argtypes = [POINTER(_RBlock), c_int, c_void_p, c_size_t, c_void_p]
        L.asteria_soap_step_workspace_bytes.restype = c_size_t
        L.asteria_soap_step_workspace_bytes.argtypes = [POINTER(_SBlock), c_int]
        L.asteria_soap_step.restype = c_int
        L.asteria_soap_step.argtypes = [POINTER(_SBlock), c_int, c_float, c_float, c_float, c_int,
                                        c_void_p, c_size_t, c_void_p]
        L.asteria_transpose.restype = c_int
        L.asteria_transpose.argtypes = [POINTER(_TPair), c_int, c_void_p]
        L.asteria_profile_enable.restype = c_int
        L.asteria_profile_enable.argtypes = [c_int]
        L.asteria_profile_collect.restype = c_int
        L.asteria_profile_collect.argtypes = [POINTER(c_float), POINTER(c_int32), c_int]
        L.asteria_packed_elems.restype = c_size_t
        L.asteria_packed_elems.argtypes = [c_int]
        for fn in (L.asteria_sym_pack, L.asteria_sym_unpack):
            fn.restype = c_int
            fn.argtypes = [POINTER(_SymPair), c_int, c_void_p]
        L.asteria_profile_i8_flops.restype = c_int
        L.asteria_profile_i8_flops.argtypes = [POINTER(ctypes.c_double)]
        _lib = L
    return _lib


def version() -> int:
    return lib().asteria_version()


def status_string(status: int) -> str:
    return lib().asteria_status_string(int(status)).decode()


# ---------------------------------------------------------------------------- marshalling

def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _mat(t: Optional[torch.Tensor], name: str, dtype=None):
    """(pointer, rows, cols, leading dimension) of a 2-D row-major device tensor."""
    if t is None:
        return None, 0, 0, 0
    if t.dim() != 2 or t.stride(1) != 1 and t.shape[1] > 1:
        raise ValueError(f"{name}: need a 2-D tensor with unit column stride")
    if not t.is_cuda:
        raise ValueError(f"{name}: need a GPU tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    ld = t.stride(0) if t.shape[0] > 1 else max(t.shape[1], t.stride(0))
    return t.data_ptr(), t.shape[0], t.shape[1], ld


def packed_elems(n: int) -> int:
    """Floats a symmetric n x n matrix occupies in packed lower tiles."""
    return lib().asteria_packed_elems(int(n))


def _packed(t: Optional[torch.Tensor], n: int, name: str):
    if t is None:
        return None
    if not t.is_cuda or t.dtype != torch.float32 or t.dim() != 1 or not t.is_contiguous() or t.numel() < packed_elems(n):
        raise ValueError(f"{name}: need a flat contiguous fp32 GPU tensor of packed_elems({n}) = {packed_elems(n)} elements")
    return t.data_ptr()


class _Batch:
    """A host descriptor array plus the tensors it points to (kept alive)."""
    ctype = None

    def __init__(self, items):
        self.items = [tuple(i) for i in items]
        self.count = len(self.items)
        self.array = (self.ctype * max(self.count, 1))()
        for k, it in enumerate(self.items):
            self._fill(self.array[k], *it)

    def __len__(self):
        return self.count


class Blocks(_Batch):
    """[(G, L, R)] or [(G, L, R, acc)] for stats_update; L or R may be None, acc is ACC_F32 (default)
    or ACC_F64."""
    ctype = _Block

    def _fill(self, d, G, L, R, acc=ACC_F32, layout=LAYOUT_FULL):
        d.acc = int(acc)
        d.lr_layout = int(layout)
        d.G, d.m, d.n, d.ldg = _mat(G, "G")
        d.g_dtype = _dtype_code(G)
        if layout == LAYOUT_PACKED:       # L, R: flat fp32 tensors of packed_elems(m), packed_elems(n)
            d.L, d.R = _packed(L, d.m, "L"), _packed(R, d.n, "R")
            d.ldl = d.ldr = 0
            return
        d.L, _, _, d.ldl = _mat(L, "L", torch.float32)
        d.R, _, _, d.ldr = _mat(R, "R", torch.float32)
        if L is not None and tuple(L.shape) != (d.m, d.m) or R is not None and tuple(R.shape) != (d.n, d.n):
            raise ValueError("L must be m x m and R n x n")


class Factors(_Batch):
    """[(A, X)] for inverse_root (X written) and soap_refresh (X = Q, in place)."""
    ctype = _Factor

    def _fill(self, d, A, X, a_layout=LAYOUT_FULL):
        d.X, xn, xn2, d.ldx = _mat(X, "X", torch.float32)
        d.a_layout = int(a_layout)
        if a_layout == LAYOUT_PACKED:     # A: flat fp32 tensor of packed_elems(n)
            if xn != xn2:
                raise ValueError("X must be square")
            d.A, d.lda, d.n = _packed(A, xn, "A"), 0, xn
            return
        d.A, n, n2, d.lda = _mat(A, "A", torch.float32)
        if n != n2 or (xn, xn2) != (n, n):
            raise ValueError("A and X must be square and of equal size")
        d.n = n


class PBlocks(_Batch):
    """[(XL, G, XR, P)] for precondition."""
    ctype = _PBlock

    def _fill(self, d, XL, G, XR, P):
        d.G, d.m, d.n, d.ldg = _mat(G, "G")
        d.g_dtype = _dtype_code(G)
        d.XL, a, b, d.ldxl = _mat(XL, "XL", torch.float32)
        d.XR, c, e, d.ldxr = _mat(XR, "XR", torch.float32)
        d.P, pm, pn, d.ldp = _mat(P, "P")
        d.p_dtype = _dtype_code(P)
        if (a, b) != (d.m, d.m) or (c, e) != (d.n, d.n) or (pm, pn) != (d.m, d.n):
            raise ValueError("shape mismatch in precondition block")


class SBlocks(_Batch):
    """[(G, QL, QR, M, V, N)] or [(G, QL, QR, M, V, N, QLt, QRt)] for soap_step; QL or QR may be None (the
    identity on that side); QLt, QRt: transposed copies of the bases kept by the caller (`transpose`), or None."""
    ctype = _SBlock

    def _fill(self, d, G, QL, QR, M, V, N, QLt=None, QRt=None):
        d.G, d.m, d.n, d.ldg = _mat(G, "G")
        d.g_dtype = _dtype_code(G)
        d.QL, a, b, d.ldql = _mat(QL, "QL", torch.float32)
        d.QR, c, e, d.ldqr = _mat(QR, "QR", torch.float32)
        d.M, m1, n1, d.ldm = _mat(M, "M", torch.float32)
        d.V, m2, n2, d.ldv = _mat(V, "V", torch.float32)
        d.N, m3, n3, d.ldn = _mat(N, "N", torch.float32)
        if (QL is not None and (a, b) != (d.m, d.m)) or (QR is not None and (c, e) != (d.n, d.n)) or \
                {(m1, n1), (m2, n2), (m3, n3)} != {(d.m, d.n)}:
            raise ValueError("shape mismatch in soap block")
        d.QLt, a, b, d.ldqlt = _mat(QLt, "QLt", torch.float32)
        d.QRt, c, e, d.ldqrt = _mat(QRt, "QRt", torch.float32)
        if (QLt is not None and (a, b) != (d.m, d.m)) or (QRt is not None and (c, e) != (d.n, d.n)):
            raise ValueError("shape mismatch in soap block (transposed bases)")


def _as(batch_type, items):
    return items if isinstance(items, batch_type) else batch_type(items)


def _stream(stream) -> c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return c_void_p(stream.cuda_stream)


def _workspace(ws: Optional[torch.Tensor], need: int, device) -> torch.Tensor:
    if ws is None:
        ws = torch.empty(max(int(need), 256), dtype=torch.uint8, device=device)
    if not ws.is_cuda or ws.dtype != torch.uint8 or not ws.is_contiguous():
        raise ValueError("workspace must be a contiguous uint8 GPU tensor")
    return ws


def _ptr(t: Optional[torch.Tensor], dtype, count, name):
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or t.numel() < count or not t.is_contiguous():
        raise ValueError(f"{name}: need a contiguous GPU tensor of {dtype} with >= {count} elements")
    return c_void_p(t.data_ptr())


def _check(st: int, where: str):
    if st != OK:
        raise AsteriaError(st, where)


# ---------------------------------------------------------------------------- entry points

def stats_update_workspace_bytes(blocks) -> int:
    b = _as(Blocks, blocks)
    return lib().asteria_stats_update_workspace_bytes(b.array, b.count)


def stats_update(blocks, beta: float, ws: Optional[torch.Tensor] = None, stream=None) -> None:
    """L <- beta L + (1-beta) G G^T, R <- beta R + (1-beta) G^T G for every (G, L, R)."""
    b = _as(Blocks, blocks)
    dev = b.items[0][0].device if b.count else None
    ws = _workspace(ws, stats_update_workspace_bytes(b), dev)
    _check(lib().asteria_stats_update(b.array, b.count, float(beta), c_void_p(ws.data_ptr()), ws.numel(),
                                      _stream(stream)), "asteria_stats_update")


def inverse_root_workspace_bytes(factors, opts: Optional[RootOpts] = None):
    """(bytes for a single pass over the whole batch, smallest accepted size)."""
    f = _as(Factors, factors)
    mn = c_size_t(0)
    full = lib().asteria_inverse_root_workspace_bytes(f.array, f.count, ctypes.byref(opts) if opts else None,
                                                      ctypes.byref(mn))
    return full, mn.value


def inverse_root_plan(eps, relative: bool = True, root: int = 4, opts: Optional[RootOpts] = None):
    """(fp64 prefix length of the M-chain, its first iteration on the fp16 matrix cores with split
    operands, whether every X update runs there) as the library would choose."""
    eps_list = [float(eps)] if not isinstance(eps, (Sequence, torch.Tensor)) else [float(e) for e in eps]
    eps_arr = (c_float * len(eps_list))(*eps_list)
    j64, jl, xt = c_int32(0), c_int32(0), c_int32(0)
    _check(lib().asteria_inverse_root_plan(int(root), EPS_RELATIVE if relative else EPS_ABSOLUTE, eps_arr,
                                           len(eps_list), ctypes.byref(opts) if opts else None,
                                           ctypes.byref(j64), ctypes.byref(jl), ctypes.byref(xt)),
           "asteria_inverse_root_plan")
    return j64.value, jl.value, bool(xt.value)


def inverse_root(factors, eps, relative: bool = True, root: int = 4, opts: Optional[RootOpts] = None,
                 info: Optional[torch.Tensor] = None, iters: Optional[torch.Tensor] = None,
                 resid: Optional[torch.Tensor] = None, lambda_max: Optional[torch.Tensor] = None,
                 ws: Optional[torch.Tensor] = None, stream=None) -> None:
    """X = (A + eps I)^(-1/root) for every (A, X).  ``eps``: float or sequence of one per factor."""
    f = _as(Factors, factors)
    eps_list = [float(eps)] if not isinstance(eps, (Sequence, torch.Tensor)) else [float(e) for e in eps]
    eps_arr = (c_float * len(eps_list))(*eps_list)
    dev = f.items[0][0].device if f.count else None
    if ws is None:
        full, _ = inverse_root_workspace_bytes(f, opts)
        ws = _workspace(None, full, dev)
    ws = _workspace(ws, 0, dev)
    st = lib().asteria_inverse_root(f.array, f.count, int(root), EPS_RELATIVE if relative else EPS_ABSOLUTE,
                                    eps_arr, len(eps_list), ctypes.byref(opts) if opts else None,
                                    _ptr(info, torch.int32, f.count, "info"),
                                    _ptr(iters, torch.int32, f.count, "iters"),
                                    _ptr(resid, torch.float32, f.count, "resid"),
                                    _ptr(lambda_max, torch.float32, f.count, "lambda_max"),
                                    c_void_p(ws.data_ptr()), ws.numel(), _stream(stream))
    _check(st, "asteria_inverse_root")


def static_scratch_bytes() -> int:
    return lib().asteria_static_scratch_bytes()


def inverse_root_static(factors, eps, relative: bool = True, root: int = 4, opts: Optional[RootOpts] = None,
                        info: Optional[torch.Tensor] = None, iters: Optional[torch.Tensor] = None,
                        resid: Optional[torch.Tensor] = None, lambda_max: Optional[torch.Tensor] = None,
                        stream=None) -> None:
    """inverse_root on the library's fixed scratch array: no workspace, no allocation anywhere."""
    f = _as(Factors, factors)
    eps_list = [float(eps)] if not isinstance(eps, (Sequence, torch.Tensor)) else [float(e) for e in eps]
    eps_arr = (c_float * len(eps_list))(*eps_list)
    st = lib().asteria_inverse_root_static(f.array, f.count, int(root),
                                           EPS_RELATIVE if relative else EPS_ABSOLUTE, eps_arr, len(eps_list),
                                           ctypes.byref(opts) if opts else None,
                                           _ptr(info, torch.int32, f.count, "info"),
                                           _ptr(iters, torch.int32, f.count, "iters"),
                                           _ptr(resid, torch.float32, f.count, "resid"),
                                           _ptr(lambda_max, torch.float32, f.count, "lambda_max"),
                                           _stream(stream))
    _check(st, "asteria_inverse_root_static")


def precondition_workspace_bytes(blocks) -> int:
    b = _as(PBlocks, blocks)
    return lib().asteria_precondition_workspace_bytes(b.array, b.count)


def precondition(blocks, ws: Optional[torch.Tensor] = None, stream=None) -> None:
    """P = X_L G X_R for every (XL, G, XR, P)."""
    b = _as(PBlocks, blocks)
    dev = b.items[0][1].device if b.count else None
    ws = _workspace(ws, precondition_workspace_bytes(b), dev)
    _check(lib().asteria_precondition(b.array, b.count, c_void_p(ws.data_ptr()), ws.numel(), _stream(stream)),
           "asteria_precondition")


def soap_refresh_workspace_bytes(factors):
    f = _as(Factors, factors)
    mn = c_size_t(0)
    full = lib().asteria_soap_refresh_workspace_bytes(f.array, f.count, ctypes.byref(mn))
    return full, mn.value


def soap_refresh(factors, info: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
                 stream=None, aux_streams=None, sort: bool = False, from_identity: bool = False, rounds: int = 1,
                 perm: Optional[torch.Tensor] = None, qt=None, qt_valid: bool = False) -> None:
    """Q <- qr(A Q).Q for every (A, Q), in place.  ``qt``: per factor a tensor that receives Q^T (or None);
    ``qt_valid``: those tensors already hold the transpose of the incoming Q.  ``aux_streams``: up to four torch streams on which
    groups of factors are enqueued side by side; ``sort``: columns ordered by decreasing q^T A q first
    (``perm``: int32 GPU tensor of sum(n) entries receiving the orders); ``from_identity`` / ``rounds``:
    start from Q = I and run several rounds (asteria_soap_refresh_ex)."""
    f = _as(Factors, factors)
    dev = f.items[0][0].device if f.count else None
    if ws is None:
        ws = _workspace(None, soap_refresh_workspace_bytes(f)[0], dev)
    ws = _workspace(ws, 0, dev)
    if not (aux_streams or sort or from_identity or rounds != 1 or perm is not None or qt is not None):
        _check(lib().asteria_soap_refresh(f.array, f.count, _ptr(info, torch.int32, f.count, "info"),
                                          c_void_p(ws.data_ptr()), ws.numel(), _stream(stream)),
               "asteria_soap_refresh")
        return
    o = SoapRefreshOpts()
    lib().asteria_soap_refresh_opts_default(ctypes.byref(o))
    o.sort, o.from_identity, o.rounds = int(bool(sort)), int(bool(from_identity)), int(rounds)
    aux = None
    if aux_streams:
        aux = (c_void_p * len(aux_streams))(*[s.cuda_stream for s in aux_streams])
        o.n_aux, o.aux_streams = len(aux_streams), ctypes.cast(aux, POINTER(c_void_p))
    xt_arr = ld_arr = None
    if qt is not None:
        qt = list(qt)
        if len(qt) != f.count:
            raise ValueError("qt: one entry per factor")
        xt_arr, ld_arr = (c_void_p * f.count)(), (c_int32 * f.count)()
        for i, t in enumerate(qt):
            ptr, r, c, ld = _mat(t, "qt", torch.float32)
            if t is not None and (r, c) != tuple(f.items[i][1].shape):
                raise ValueError("qt: shape of the basis expected")
            xt_arr[i], ld_arr[i] = ptr, ld
        o.Xt, o.ldxt, o.xt_in = ctypes.cast(xt_arr, POINTER(c_void_p)), ctypes.cast(ld_arr, POINTER(c_int32)), int(bool(qt_valid))
    total = sum(it[0].shape[0] for it in f.items)
    _check(lib().asteria_soap_refresh_ex(f.array, f.count, ctypes.byref(o), _ptr(info, torch.int32, f.count, "info"),
                                         _ptr(perm, torch.int32, total, "perm"), c_void_p(ws.data_ptr()), ws.numel(),
                                         _stream(stream)), "asteria_soap_refresh_ex")


class RBlocks(_Batch):
    """[(QL_old, QL_new, QR_old, QR_new, M, V, permL, permR)] for soap_reproject; M, V, permL, permR may be None."""
    ctype = _RBlock

    def _fill(self, d, QLo, QLn, QRo, QRn, M, V=None, permL=None, permR=None):
        ref = M if M is not None else V
        d.m, d.n = ref.shape
        d.M, _, _, d.ldm = _mat(M, "M", torch.float32)
        d.V, _, _, d.ldv = _mat(V, "V", torch.float32)
        d.QL_old, a, b, d.ldql_old = _mat(QLo, "QL_old", torch.float32)
        d.QL_new, a2, b2, d.ldql_new = _mat(QLn, "QL_new", torch.float32)
        d.QR_old, c, e, d.ldqr_old = _mat(QRo, "QR_old", torch.float32)
        d.QR_new, c2, e2, d.ldqr_new = _mat(QRn, "QR_new", torch.float32)
        if M is not None and not ((a, b) == (a2, b2) == (d.m, d.m) and (c, e) == (c2, e2) == (d.n, d.n)):
            raise ValueError("shape mismatch in reproject block")
        d.permL = _ptr(permL, torch.int32, d.m, "permL")
        d.permR = _ptr(permR, torch.int32, d.n, "permR")


def soap_reproject_workspace_bytes(blocks) -> int:
    b = _as(RBlocks, blocks)
    return lib().asteria_soap_reproject_workspace_bytes(b.array, b.count)


def soap_reproject(blocks, ws: Optional[torch.Tensor] = None, stream=None) -> None:
    """M <- QL_new^T (QL_old M QR_old^T) QR_new and V[i][j] <- V[permL[i]][permR[j]] for every block."""
    b = _as(RBlocks, blocks)
    ref = next(t for t in b.items[0] if t is not None)
    ws = _workspace(ws, soap_reproject_workspace_bytes(b), ref.device)
    _check(lib().asteria_soap_reproject(b.array, b.count, c_void_p(ws.data_ptr()), ws.numel(), _stream(stream)),
           "asteria_soap_reproject")


def soap_step_workspace_bytes(blocks) -> int:
    b = _as(SBlocks, blocks)
    return lib().asteria_soap_step_workspace_bytes(b.array, b.count)


def soap_step(blocks, beta1: float, beta2: float, adam_eps: float, step_t: int,
              ws: Optional[torch.Tensor] = None, stream=None) -> None:
    """N = Q_L Adam(Q_L^T G Q_R) Q_R^T for every (G, QL, QR, M, V, N); M, V updated in place."""
    b = _as(SBlocks, blocks)
    dev = b.items[0][0].device if b.count else None
    ws = _workspace(ws, soap_step_workspace_bytes(b), dev)
    _check(lib().asteria_soap_step(b.array, b.count, float(beta1), float(beta2), float(adam_eps), int(step_t),
                                   c_void_p(ws.data_ptr()), ws.numel(), _stream(stream)), "asteria_soap_step")


def transpose(pairs, stream=None) -> None:
    """dst = src^T for every (src, dst) pair of fp32 device matrices (what soap_step takes as QLt, QRt)."""
    pairs = list(pairs)
    arr = (_TPair * len(pairs))()
    for d, (src, dst) in zip(arr, pairs):
        d.src, d.rows, d.cols, d.lds = _mat(src, "src", torch.float32)
        d.dst, r2, c2, d.ldd = _mat(dst, "dst", torch.float32)
        if (r2, c2) != (d.cols, d.rows):
            raise ValueError("dst must have the transposed shape")
    _check(lib().asteria_transpose(arr, len(pairs), _stream(stream)), "asteria_transpose")


def profile_enable(max_launches: int = 4096) -> None:
    """Start bracketing every grouped-GEMM launch with HIP events (measurement aid)."""
    _check(lib().asteria_profile_enable(int(max_launches)), "asteria_profile_enable")


def profile_collect(cap: int = 4096):
    """Stop recording; returns [(milliseconds, kind)] per launch in launch order."""
    ms = (c_float * cap)()
    kind = (c_int32 * cap)()
    n = lib().asteria_profile_collect(ms, kind, cap)
    if n < 0:
        raise AsteriaError(INVALID_ARG, "asteria_profile_collect")
    return [(ms[i], kind[i]) for i in range(n)]


def profile_i8_flops():
    """Algorithmic flops of the fp64 iterations' products since profile_enable, by where they ran:
    (fp64 cores, int8 cores with 4 slices, int8 cores with 5 slices).  Waits for the device."""
    out = (ctypes.c_double * 3)()
    _check(lib().asteria_profile_i8_flops(out), "asteria_profile_i8_flops")
    return tuple(out)


def _sympairs(items):
    arr = (_SymPair * max(len(items), 1))()
    for k, (full, packed) in enumerate(items):
        arr[k].full, n, n2, arr[k].ld = _mat(full, "full", torch.float32)
        if n != n2:
            raise ValueError("full: need a square matrix")
        arr[k].n = n
        arr[k].packed = _packed(packed, n, "packed")
    return arr


def sym_pack(items, stream=None) -> None:
    """packed <- lower tiles of full, for every (full, packed)."""
    _check(lib().asteria_sym_pack(_sympairs(items), len(items), _stream(stream)), "asteria_sym_pack")


def sym_unpack(items, stream=None) -> None:
    """full <- packed (both triangles), for every (full, packed)."""
    _check(lib().asteria_sym_unpack(_sympairs(items), len(items), _stream(stream)), "asteria_sym_unpack")
