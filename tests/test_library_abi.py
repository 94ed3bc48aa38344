"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and rejects bad arguments on the host before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import pytest

import paper_2605_16184_amd as ast
from paper_2605_16184_amd import binding as B
from paper_2605_16184_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "asteria.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(asteria_[a-z0-9_]+)\s*\(", hdr))
    assert {"asteria_stats_update", "asteria_inverse_root", "asteria_precondition", "asteria_soap_refresh",
            "asteria_soap_step"} <= names
    lib = ast.lib()
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in asteria.h but not exported"


def test_version_status_strings_and_default_options():
    assert ast.version() >= 100
    assert ast.status_string(B.OK) == "ok"
    assert "workspace" in ast.status_string(B.WORKSPACE_TOO_SMALL)
    o = ast.RootOpts()
    assert (o.max_iters, o.fp64_iters, o.power_iters, o.schedule) == (40, -1, 256, 1)
    assert abs(o.stop_resid - 1e-2) < 1e-9 and abs(o.power_tol - 1e-3) < 1e-9 and abs(o.lambda_margin - 0.01) < 1e-9


def _blk(**kw):
    b = B._Block()
    b.G, b.L, b.R = 0x1000, 0x2000, 0x3000
    b.m = b.n = 8
    b.ldg = b.ldl = b.ldr = 8
    b.g_dtype = B.F32
    for k, v in kw.items():
        setattr(b, k, v)
    return (B._Block * 1)(b)


def test_stats_update_rejects_bad_arguments_without_launching():
    f = ast.lib().asteria_stats_update
    ws = ctypes.c_void_p(0x10000)
    assert f(None, 1, 0.9, ws, 1 << 20, None) == B.INVALID_ARG
    assert f(_blk(), 0, 0.9, ws, 1 << 20, None) == B.INVALID_ARG
    assert f(_blk(), 1, 1.0, ws, 1 << 20, None) == B.INVALID_ARG
    assert f(_blk(), 1, -0.1, ws, 1 << 20, None) == B.INVALID_ARG
    assert f(_blk(G=None), 1, 0.9, ws, 1 << 20, None) == B.INVALID_ARG
    assert f(_blk(m=0), 1, 0.9, ws, 1 << 20, None) == B.INVALID_ARG
    assert f(_blk(ldg=7), 1, 0.9, ws, 1 << 20, None) == B.INVALID_ARG
    assert f(_blk(ldl=7), 1, 0.9, ws, 1 << 20, None) == B.INVALID_ARG
    assert f(_blk(g_dtype=5), 1, 0.9, ws, 1 << 20, None) == B.INVALID_ARG
    assert f(_blk(acc=2), 1, 0.9, ws, 1 << 20, None) == B.INVALID_ARG
    assert f(_blk(lr_layout=2), 1, 0.9, ws, 1 << 20, None) == B.INVALID_ARG
    assert f(_blk(lr_layout=1, L=0x2004), 1, 0.9, ws, 1 << 20, None) == B.INVALID_ARG    # packed tiles: 16-byte aligned
    assert f(_blk(L=None, R=None), 1, 0.9, ws, 1 << 20, None) == B.INVALID_ARG
    assert f(_blk(), 1, 0.9, None, 0, None) == B.WORKSPACE_TOO_SMALL
    assert f(_blk(), 1, 0.9, ws, 16, None) == B.WORKSPACE_TOO_SMALL
    assert f(_blk(), 1, 0.9, ctypes.c_void_p(0x10010), 1 << 20, None) == B.INVALID_ARG   # misaligned workspace


def _fac(**kw):
    a = B._Factor()
    a.A, a.X, a.n, a.lda, a.ldx = 0x1000, 0x2000, 8, 8, 8
    for k, v in kw.items():
        setattr(a, k, v)
    return (B._Factor * 1)(a)


def test_inverse_root_rejects_bad_arguments_without_launching():
    f = ast.lib().asteria_inverse_root
    eps = (ctypes.c_float * 1)(1e-6)
    ws = ctypes.c_void_p(0x10000)
    args = lambda fac=_fac(), n=1, root=4, mode=0, e=eps, ec=1, opts=None, w=ws, wb=1 << 30: (
        fac, n, root, mode, e, ec, opts, None, None, None, None, w, wb, None)
    assert f(*args(fac=None)) == B.INVALID_ARG
    assert f(*args(n=0)) == B.INVALID_ARG
    assert f(*args(root=3)) == B.UNSUPPORTED
    assert f(*args(root=8)) == B.UNSUPPORTED
    assert f(*args(mode=7)) == B.INVALID_ARG
    assert f(*args(e=None)) == B.INVALID_ARG
    assert f(*args(ec=2)) == B.INVALID_ARG
    assert f(*args(e=(ctypes.c_float * 1)(-1.0))) == B.INVALID_ARG
    assert f(*args(e=(ctypes.c_float * 1)(float("nan")))) == B.INVALID_ARG
    assert f(*args(fac=_fac(A=None))) == B.INVALID_ARG
    assert f(*args(fac=_fac(n=-1))) == B.INVALID_ARG
    assert f(*args(fac=_fac(lda=4))) == B.INVALID_ARG
    bad = ast.RootOpts(max_iters=0)
    assert f(*args(opts=ctypes.byref(bad))) == B.INVALID_ARG
    bad = ast.RootOpts(schedule=9)
    assert f(*args(opts=ctypes.byref(bad))) == B.UNSUPPORTED
    assert f(*args(w=None)) == B.WORKSPACE_TOO_SMALL
    assert f(*args(wb=64)) == B.WORKSPACE_TOO_SMALL


def test_precondition_and_soap_reject_bad_arguments_without_launching():
    lib = ast.lib()
    ws = ctypes.c_void_p(0x10000)
    p = B._PBlock()
    p.XL, p.G, p.XR, p.P = 0x1000, 0x2000, 0x3000, 0x4000
    p.m, p.n, p.ldxl, p.ldg, p.ldxr, p.ldp = 4, 6, 4, 6, 6, 6
    arr = (B._PBlock * 1)(p)
    assert lib.asteria_precondition(arr, 1, None, 0, None) == B.WORKSPACE_TOO_SMALL
    p.ldp = 5
    assert lib.asteria_precondition((B._PBlock * 1)(p), 1, ws, 1 << 20, None) == B.INVALID_ARG
    p.ldp = 6
    p.p_dtype = 3
    assert lib.asteria_precondition((B._PBlock * 1)(p), 1, ws, 1 << 20, None) == B.INVALID_ARG
    assert lib.asteria_precondition(None, 1, ws, 1 << 20, None) == B.INVALID_ARG

    t = B._TPair()
    t.src, t.dst, t.rows, t.cols, t.lds, t.ldd = 0x1000, 0x2000, 4, 6, 6, 3
    assert lib.asteria_transpose((B._TPair * 1)(t), 1, None) == B.INVALID_ARG          # ldd < rows
    t.ldd, t.dst = 4, None
    assert lib.asteria_transpose((B._TPair * 1)(t), 1, None) == B.INVALID_ARG
    assert lib.asteria_transpose(None, 1, None) == B.INVALID_ARG

    s = B._SBlock()
    s.G, s.QL, s.QR, s.M, s.V, s.N = 0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000
    s.m, s.n = 4, 6
    s.ldg = s.ldqr = s.ldm = s.ldv = s.ldn = 6
    s.ldql = 4
    one = (B._SBlock * 1)(s)
    assert lib.asteria_soap_step(one, 1, 0.9, 0.95, 1e-8, 0, ws, 1 << 20, None) == B.INVALID_ARG   # t >= 1
    assert lib.asteria_soap_step(one, 1, 1.0, 0.95, 1e-8, 1, ws, 1 << 20, None) == B.INVALID_ARG
    assert lib.asteria_soap_step(one, 1, 0.9, 0.95, 1e-8, 1, None, 0, None) == B.WORKSPACE_TOO_SMALL
    s.ldql = 3
    assert lib.asteria_soap_step((B._SBlock * 1)(s), 1, 0.9, 0.95, 1e-8, 1, ws, 1 << 20, None) == B.INVALID_ARG
    s.ldql = 4
    s.QLt, s.ldqlt = 0x9000, 3                   # a kept transpose needs its leading dimension too
    assert lib.asteria_soap_step((B._SBlock * 1)(s), 1, 0.9, 0.95, 1e-8, 1, ws, 1 << 20, None) == B.INVALID_ARG
    s.QLt, s.ldqlt, s.ldql = None, 0, 3
    s.QL = None                                  # one-sided block: the leading dimension of the absent basis is not looked at
    assert lib.asteria_soap_step((B._SBlock * 1)(s), 1, 0.9, 0.95, 1e-8, 1, None, 0, None) == B.WORKSPACE_TOO_SMALL
    s.QR = None                                  # ... but both absent is plain Adam, not this call
    assert lib.asteria_soap_step((B._SBlock * 1)(s), 1, 0.9, 0.95, 1e-8, 1, ws, 1 << 20, None) == B.INVALID_ARG
    assert lib.asteria_soap_refresh(None, 1, None, ws, 1 << 20, None) == B.INVALID_ARG
    assert lib.asteria_soap_refresh(_fac(ldx=2), 1, None, ws, 1 << 20, None) == B.INVALID_ARG
    assert lib.asteria_soap_refresh(_fac(), 1, None, None, 0, None) == B.WORKSPACE_TOO_SMALL
    assert lib.asteria_soap_refresh(_fac(), 1, None, ws, 128, None) == B.WORKSPACE_TOO_SMALL
    # extended call: auxiliary streams (at most four, none null, none equal to the caller's stream), options
    ex = lib.asteria_soap_refresh_ex
    s1, s2 = ctypes.c_void_p(0x5000), ctypes.c_void_p(0x6000)
    def opts(**kw):
        o = B.SoapRefreshOpts()
        lib.asteria_soap_refresh_opts_default(ctypes.byref(o))
        assert (o.sort, o.from_identity, o.rounds, o.n_aux) == (0, 0, 1, 0)
        for k, v in kw.items():
            setattr(o, k, v)
        return ctypes.byref(o)
    two = ctypes.cast((ctypes.c_void_p * 2)(s1, s2), ctypes.POINTER(ctypes.c_void_p))
    bad = ctypes.cast((ctypes.c_void_p * 2)(s1, None), ctypes.POINTER(ctypes.c_void_p))
    assert ex(_fac(), 1, opts(n_aux=5, aux_streams=two), None, None, ws, 1 << 20, None) == B.INVALID_ARG
    assert ex(_fac(), 1, opts(n_aux=2), None, None, ws, 1 << 20, None) == B.INVALID_ARG
    assert ex(_fac(), 1, opts(n_aux=2, aux_streams=two), None, None, ws, 1 << 20, s1) == B.INVALID_ARG
    assert ex(_fac(), 1, opts(n_aux=2, aux_streams=bad), None, None, ws, 1 << 20, None) == B.INVALID_ARG
    assert ex(None, 1, opts(n_aux=2, aux_streams=two), None, None, ws, 1 << 20, None) == B.INVALID_ARG
    assert ex(_fac(), 1, opts(n_aux=2, aux_streams=two), None, None, ws, 128, None) == B.WORKSPACE_TOO_SMALL
    assert ex(_fac(), 1, opts(sort=2), None, None, ws, 1 << 20, None) == B.INVALID_ARG
    assert ex(_fac(), 1, opts(rounds=0), None, None, ws, 1 << 20, None) == B.INVALID_ARG
    perm = ctypes.c_void_p(0x7000)
    assert ex(_fac(), 1, opts(), None, perm, ws, 1 << 20, None) == B.INVALID_ARG               # an order without sorting
    assert ex(_fac(), 1, opts(sort=1, rounds=2), None, perm, ws, 1 << 20, None) == B.INVALID_ARG
    # buffers for Q^T: pointers and leading dimensions come together, a buffer is not Q itself, ld >= n
    xt = ctypes.cast((ctypes.c_void_p * 1)(0x8000), ctypes.POINTER(ctypes.c_void_p))
    xq = ctypes.cast((ctypes.c_void_p * 1)(0x2000), ctypes.POINTER(ctypes.c_void_p))
    ld8 = ctypes.cast((ctypes.c_int32 * 1)(8), ctypes.POINTER(ctypes.c_int32))
    ld7 = ctypes.cast((ctypes.c_int32 * 1)(7), ctypes.POINTER(ctypes.c_int32))
    assert ex(_fac(), 1, opts(Xt=xt), None, None, ws, 1 << 20, None) == B.INVALID_ARG
    assert ex(_fac(), 1, opts(Xt=xt, ldxt=ld7), None, None, ws, 1 << 20, None) == B.INVALID_ARG
    assert ex(_fac(), 1, opts(Xt=xq, ldxt=ld8), None, None, ws, 1 << 20, None) == B.INVALID_ARG
    assert ex(_fac(), 1, opts(Xt=xt, ldxt=ld8, xt_in=2), None, None, ws, 1 << 20, None) == B.INVALID_ARG
    assert ex(_fac(), 1, opts(Xt=xt, ldxt=ld8, xt_in=1), None, None, ws, 128, None) == B.WORKSPACE_TOO_SMALL
    # re-projection of the moments
    rp = lib.asteria_soap_reproject
    def rblk(**kw):
        r = B._RBlock()
        r.QL_old, r.QL_new, r.QR_old, r.QR_new, r.M, r.V = 0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000
        r.m = r.n = 8
        r.ldql_old = r.ldql_new = r.ldqr_old = r.ldqr_new = r.ldm = r.ldv = 8
        for k, v in kw.items():
            setattr(r, k, v)
        return (B._RBlock * 1)(r)
    assert rp(None, 1, ws, 1 << 20, None) == B.INVALID_ARG
    assert rp(rblk(m=0), 1, ws, 1 << 20, None) == B.INVALID_ARG
    assert rp(rblk(M=None, V=None), 1, ws, 1 << 20, None) == B.INVALID_ARG
    assert rp(rblk(QL_new=None), 1, ws, 1 << 20, None) == B.INVALID_ARG
    assert rp(rblk(ldm=7), 1, ws, 1 << 20, None) == B.INVALID_ARG
    assert rp(rblk(ldv=7), 1, ws, 1 << 20, None) == B.INVALID_ARG
    assert rp(rblk(), 1, ws, 64, None) == B.WORKSPACE_TOO_SMALL
    assert lib.asteria_soap_reproject_workspace_bytes(rblk(), 1) > 0


def test_workspace_queries_scale_with_the_batch():
    one = _fac(n=1024, lda=1024, ldx=1024)
    mn = ctypes.c_size_t(0)
    full = ast.lib().asteria_inverse_root_workspace_bytes(one, 1, None, ctypes.byref(mn))
    # default options reserve 2 fp32 and 4 fp64 work matrices per factor (X stays in fp32 in every
    # tier; the fp32 matrices of the M-chain reuse the room of the fp64 T and T^4) and two operands
    # of 5 int8 slices
    assert full >= (2 * 4 + 4 * 8 + 2 * 5) * 1024 * 1024 and full < 1.1 * (2 * 4 + 4 * 8 + 2 * 5) * 1024 * 1024
    assert mn.value == full
    o = ast.RootOpts(int8_slices=0)
    f64 = ast.lib().asteria_inverse_root_workspace_bytes(one, 1, ctypes.byref(o), None)
    assert (2 * 4 + 4 * 8) * 1024 * 1024 <= f64 < 1.1 * (2 * 4 + 4 * 8) * 1024 * 1024
    o = ast.RootOpts(fp64_iters=0)
    f32 = ast.lib().asteria_inverse_root_workspace_bytes(one, 1, ctypes.byref(o), None)
    assert 5 * 4 * 1024 * 1024 <= f32 < 1.1 * 5 * 4 * 1024 * 1024
    assert ast.lib().asteria_inverse_root_workspace_bytes(None, 1, None, None) == 0


def test_precision_plan_follows_eps_and_pinned_options():
    # host logic only: which leading iterations keep fp64, where the split-fp16 tier starts, and
    # whether the X updates run there from the first product on
    assert ast.inverse_root_plan(1e-6) == (2, 2, True)          # the headline setting: 2 fp64 iterations, no fp32 tier
    j64, jl, xt = ast.inverse_root_plan(1e-8)
    assert j64 == jl and 3 <= j64 <= 5 and xt                    # a smaller eps keeps fp64 longer
    j64b, jlb, _ = ast.inverse_root_plan(1e-2)
    assert j64b == 0 and jlb == 0                                # well above fp32 round-off: no fp64 at all
    o = ast.RootOpts()
    j64a, jla, xta = ast.inverse_root_plan(1e-6, relative=False)
    assert jla >= o.max_iters and not xta                        # absolute eps: the host cannot place the spectrum
    assert ast.inverse_root_plan(1e-6, opts=ast.RootOpts(fp64_iters=0))[::2] == (0, False)   # pinned: X follows M's tier
    assert ast.inverse_root_plan(1e-6, opts=ast.RootOpts(lowp_from=5))[1:] == (5, False)
    # the fp64 prefix and the start of the 16-bit tier follow one rule from one start of the interval
    # (half of eps s, as on the device): under the automatic rules they coincide for every eps
    for e in (3e-1, 1e-2, 3e-4, 1e-4, 3e-5, 1e-5, 3e-6, 1e-6, 3e-7, 1e-7, 3e-8, 1e-8, 1e-9, 1e-10):
        for sched in (1, 0):
            j, l, _ = ast.inverse_root_plan(e, opts=ast.RootOpts(schedule=sched))
            assert j == l, (e, sched, j, l)
    j64c, _, _ = ast.inverse_root_plan(1e-6, opts=ast.RootOpts(schedule=0))
    assert j64c > 2                                              # classical coefficients lift the spectrum more slowly
    # where the products of the fp64 iterations run is a separate option: default (int8 cores, up to 5
    # slices), fp64 cores, at most 4 slices; other counts are refused
    assert ast.RootOpts().int8_slices == -1
    for ns in (0, 4, 5):
        assert ast.inverse_root_plan(1e-6, opts=ast.RootOpts(int8_slices=ns)) == (2, 2, True)
    eps1 = (ctypes.c_float * 1)(1e-6)
    for ns in (3, 6, -2):
        o = ast.RootOpts(int8_slices=ns)
        assert ast.lib().asteria_inverse_root_plan(4, 0, eps1, 1, ctypes.byref(o), None, None, None) == B.UNSUPPORTED


def test_model_block_census_matches_the_1p1b_configuration():
    mats = W.llama_1b_matrices()
    blocks = W.block_shapes(mats, 1024)
    by_shape, by_factor, params = W.census(blocks)
    assert params == 1_099_956_224 and len(blocks) == 1184
    assert by_shape == {(1024, 1024): 960, (256, 1024): 92, (512, 1024): 88, (1024, 512): 44}
    assert by_factor == {1024: 2144, 512: 132, 256: 92}
    blocks = W.block_shapes(mats, 2048)
    by_shape, by_factor, params = W.census(blocks)
    assert len(blocks) == 318 and by_factor == {2048: 524, 1536: 66, 1280: 2, 256: 44}
    assert W.split_dim(5632, 1024) == [1024] * 5 + [512] and W.split_dim(32000, 2048)[-1] == 1280


def test_generators_are_seeded_and_shaped():
    import torch
    a = W.lowrank_block(64, 48, "cpu", 1, 2)
    b = W.lowrank_block(64, 48, "cpu", 1, 2)
    c = W.lowrank_block(64, 48, "cpu", 1, 3)
    assert a.dtype == torch.bfloat16 and a.shape == (64, 48)
    assert torch.equal(a, b) and not torch.equal(a, c)
    q = W.haar(32, "cpu", 0, dtype=torch.float64)
    assert q.is_contiguous() and torch.allclose(q.T @ q, torch.eye(32, dtype=torch.float64), atol=1e-12)
    g = W.spectrum_block(q, q, W.powerlaw_sigma(32, "cpu"), "cpu", 9, rms=None, dtype=torch.float64)
    s = torch.linalg.svdvals(g)
    assert torch.allclose(s, W.powerlaw_sigma(32, "cpu"), atol=1e-12)


def test_binding_refuses_cpu_tensors_and_wrong_shapes():
    import torch
    G = torch.zeros(4, 6)
    with pytest.raises(ValueError):
        ast.Blocks([(G, torch.zeros(4, 4), torch.zeros(6, 6))])


def test_packed_storage_sizes_and_argument_checks():
    assert ast.packed_elems(1) == 128 * 128 and ast.packed_elems(128) == 128 * 128
    assert ast.packed_elems(129) == 3 * 128 * 128 and ast.packed_elems(1024) == 36 * 128 * 128
    assert ast.packed_elems(0) == 0
    lib = ast.lib()
    pair = B._SymPair()
    pair.full, pair.packed, pair.n, pair.ld = 0x1000, 0x2000, 8, 8
    arr = (B._SymPair * 1)(pair)
    for fn in (lib.asteria_sym_pack, lib.asteria_sym_unpack):
        assert fn(None, 1, None) == B.INVALID_ARG
        assert fn(arr, 0, None) == B.INVALID_ARG
        for field, bad in (("full", None), ("packed", None), ("n", 0), ("ld", 7), ("packed", 0x2004)):
            q = B._SymPair()
            q.full, q.packed, q.n, q.ld = 0x1000, 0x2000, 8, 8
            setattr(q, field, bad)
            assert fn((B._SymPair * 1)(q), 1, None) == B.INVALID_ARG, field
    # a packed statistic cannot feed the eigenbasis refresh (A is a product operand there)
    fac = _fac(a_layout=1)
    assert lib.asteria_soap_refresh(fac, 1, None, ctypes.c_void_p(0x10000), 1 << 30, None) == B.UNSUPPORTED
    assert lib.asteria_inverse_root(_fac(a_layout=2), 1, 4, 0, (ctypes.c_float * 1)(1e-6), 1, None, None, None, None, None,
                                    ctypes.c_void_p(0x10000), 1 << 30, None) == B.INVALID_ARG
