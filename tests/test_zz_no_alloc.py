"""asteria_inverse_root_static (the entry point for callers that cannot allocate: its workspace is
a fixed array in the library's device image) against asteria_inverse_root on a caller workspace:
same kernels, same arithmetic, so the results must be bit-identical; two calls in a row on the
same GPU, the second with a smaller input, share the array and its leftover contents."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2605_16184_amd as ast
from paper_2605_16184_amd import binding as B
from paper_2605_16184_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _factor(n, *key):
    U = W.haar(n, DEV, *key, dtype=torch.float64)
    lam = 0.05 * W.powerlaw_sigma(n, DEV) ** 2
    A = (U * lam) @ U.T
    return (0.5 * (A + A.T)).float().contiguous()


def _both(As, eps):
    k = len(As)
    out = []
    for static in (False, True):
        Xs = [torch.full_like(A, float("nan")) for A in As]
        info = torch.full((k,), -1, dtype=torch.int32, device=DEV)
        iters = torch.full((k,), -1, dtype=torch.int32, device=DEV)
        resid = torch.zeros(k, device=DEV)
        lmax = torch.zeros(k, device=DEV)
        fn = ast.inverse_root_static if static else ast.inverse_root
        fn(list(zip(As, Xs)), eps, info=info, iters=iters, resid=resid, lambda_max=lmax)
        torch.cuda.synchronize()
        out.append((Xs, info.cpu(), iters.cpu(), resid.cpu(), lmax.cpu()))
    return out


def test_static_scratch_entry_point_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    assert ast.static_scratch_bytes() == 64 << 20
    # first call: several passes over the array (one 1024 factor fills it), ragged sizes, three precision tiers
    first = [_factor(1024, 1), _factor(300, 2), _factor(129, 3), _factor(512, 4)]
    # second call: smaller input on the dirty array
    second = [_factor(200, 5), _factor(64, 6)]
    for As, eps in ((first, 1e-6), (second, 1e-8)):
        (Xw, iw, kw, rw, lw), (Xs, is_, ks, rs, ls) = _both(As, eps)
        assert torch.all(iw == 0) and torch.equal(iw, is_) and torch.equal(kw, ks)
        assert torch.equal(rw, rs) and torch.equal(lw, ls)
        for a, b in zip(Xw, Xs):
            assert torch.equal(a, b)                      # same kernels on another buffer: bit-identical


def test_static_scratch_entry_point_rejects_a_factor_that_does_not_fit():
    n = 2048                                              # 50 B per element: 200 MiB > 64 MiB
    A = torch.eye(n, device=DEV); X = torch.empty_like(A)
    with pytest.raises(ast.AsteriaError) as e:
        ast.inverse_root_static([(A, X)], 1e-6)
    assert e.value.status == B.EXCEEDS_STATIC_SCRATCH
    # bad arguments are refused before anything else, as in the workspace entry point
    f = ast.lib().asteria_inverse_root_static
    eps = (ctypes.c_float * 1)(1e-6)
    assert f(None, 1, 4, 0, eps, 1, None, None, None, None, None, None) == B.INVALID_ARG
