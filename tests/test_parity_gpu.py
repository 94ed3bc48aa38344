"""GPU parity tests: every entry point of the C ABI is compared, stage by stage, with the
float64 CPU oracle fed exactly the arrays the GPU call consumed.

Tolerances (relative Frobenius error):
  statistics                <= 1e-5   (fp32 accumulation of exact bf16 products + fp32 EMA)
  inverse roots             <= 2e-3
  preconditioned gradients  <= 1e-2   (also SOAP updates)
  eigenbasis                ||Q^T Q - I||_F / sqrt(n) <= 1e-5, backward error <= 1e-5
"""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2605_16184_amd as ast
from paper_2605_16184_amd import binding as B
from paper_2605_16184_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL_STATS, TOL_ROOT, TOL_PRECOND = 1e-5, 2e-3, 1e-2
DEV = "cuda"


def np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float32).double().numpy()


def relF(a, b) -> float:
    a = np64(a) if isinstance(a, torch.Tensor) else np.asarray(a)
    b = np64(b) if isinstance(b, torch.Tensor) else np.asarray(b)
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


def padded(rows: int, cols: int, pad: int, dtype=torch.float32, fill=None) -> torch.Tensor:
    """rows x cols view into a (cols + pad)-wide buffer; the pad columns hold a sentinel."""
    buf = torch.full((rows, cols + pad), -777.0 if fill is None else fill, device=DEV, dtype=dtype)
    return buf[:, :cols]


def spd(n: int, *key: int) -> torch.Tensor:
    a = W.gaussian_block(n, n, 1.0, DEV, 99, *key)
    s = a @ a.T / n
    return (0.5 * (s + s.T)).contiguous()


def powerlaw_factor(n: int, *key: int) -> torch.Tensor:
    """fp32 statistic with eigenvalues (1/i)^2 (times the EMA weight 0.05), built in fp64."""
    U = W.haar(n, DEV, *key, dtype=torch.float64)
    lam = 0.05 * W.powerlaw_sigma(n, DEV) ** 2
    A = (U * lam) @ U.T
    return (0.5 * (A + A.T)).float().contiguous()


def logspaced_factor(n: int, decades: float, *key: int) -> torch.Tensor:
    U = W.haar(n, DEV, *key, dtype=torch.float64)
    lam = 0.05 * W.logspaced_sigma(n, decades, DEV) ** 2
    A = (U * lam) @ U.T
    return (0.5 * (A + A.T)).float().contiguous()


def run_roots(As, eps, relative=True, root=4, opts=None, ws=None):
    Xs = [torch.full_like(A, float("nan")) for A in As]
    k = len(As)
    info = torch.full((k,), -1, dtype=torch.int32, device=DEV)
    iters = torch.full((k,), -1, dtype=torch.int32, device=DEV)
    resid = torch.zeros(k, device=DEV)
    lmax = torch.zeros(k, device=DEV)
    ast.inverse_root(list(zip(As, Xs)), eps, relative=relative, root=root, opts=opts, info=info, iters=iters,
                     resid=resid, lambda_max=lmax, ws=ws)
    torch.cuda.synchronize()
    return Xs, info.cpu().numpy(), iters.cpu().numpy(), resid.cpu().numpy(), lmax.cpu().numpy()


# =============================================================================== a1 statistics

def test_stats_single_fp32_block_eight_ema_updates_from_identity():
    n = 128
    L = torch.eye(n, device=DEV); R = torch.eye(n, device=DEV)
    Lo, Ro = np.eye(n), np.eye(n)
    for k in range(8):
        G = W.gaussian_block(n, n, 0.01, DEV, 1, k)
        Lin, Rin = np64(L), np64(R)
        ast.stats_update([(G, L, R)], 0.95)
        torch.cuda.synchronize()
        Ls, Rs = oracle.stats_update(np64(G), Lin, Rin, 0.95)       # stage-wise: same inputs
        assert relF(L, Ls) <= TOL_STATS and relF(R, Rs) <= TOL_STATS
        Lo, Ro = oracle.stats_update(np64(G), Lo, Ro, 0.95)          # chained float64 pipeline
    assert relF(L, Lo) <= TOL_STATS and relF(R, Ro) <= TOL_STATS
    assert torch.equal(L, L.T) and torch.equal(R, R.T)


def test_stats_ragged_batch_bf16_and_fp32_with_padded_leading_dimensions():
    shapes = [(200, 328, torch.bfloat16), (1, 1, torch.float32), (3, 5, torch.bfloat16), (130, 257, torch.float32),
              (256, 1024, torch.bfloat16), (129, 127, torch.bfloat16)]
    items, refs = [], []
    for i, (m, n, dt) in enumerate(shapes):
        G = padded(m, n, 3 if i % 2 else 0, dt, fill=5.0)
        G.copy_(W.gaussian_block(m, n, 0.1, DEV, 2, i, dtype=dt))
        L = padded(m, m, 5); L.copy_(spd(m, 1, i))
        R = padded(n, n, 0); R.copy_(spd(n, 2, i))
        refs.append(oracle.stats_update(np64(G), np64(L), np64(R), 0.9))
        items.append((G, L, R))
    ast.stats_update(items, 0.9)
    torch.cuda.synchronize()
    for (G, L, R), (Lo, Ro) in zip(items, refs):
        assert relF(L, Lo) <= TOL_STATS and relF(R, Ro) <= TOL_STATS
        assert torch.equal(L, L.T) and torch.equal(R, R.T)
        assert torch.all(L._base[:, L.shape[1]:] == -777.0)     # pad columns untouched


def test_stats_whole_tile_bf16_blocks_read_in_place_or_through_the_transposed_copy():
    # G^T G of a 16-byte aligned bf16 block with whole tiles reads G in place (k-major operands);
    # the same shapes with an odd leading dimension take the transposed copy: both in one call
    shapes = [(64, 128), (192, 384), (512, 256), (128, 128), (320, 640)]
    items, refs = [], []
    for i, (m, n) in enumerate(shapes):
        for pad in (8, 3, 0):
            G = padded(m, n, pad, torch.bfloat16, fill=5.0)
            G.copy_(W.gaussian_block(m, n, 0.1, DEV, 4, i, dtype=torch.bfloat16))
            L = padded(m, m, 4); L.copy_(spd(m, 5, i))
            R = padded(n, n, 1); R.copy_(spd(n, 6, i))
            refs.append(oracle.stats_update(np64(G), np64(L), np64(R), 0.9))
            items.append((G, L, R))
    ast.stats_update(items, 0.9)
    torch.cuda.synchronize()
    for (G, L, R), (Lo, Ro) in zip(items, refs):
        assert relF(L, Lo) <= TOL_STATS and relF(R, Ro) <= TOL_STATS, (tuple(G.shape), relF(L, Lo), relF(R, Ro))
        assert torch.equal(L, L.T) and torch.equal(R, R.T)
        assert torch.all(R._base[:, R.shape[1]:] == -777.0) and torch.all(G._base[:, G.shape[1]:] == 5.0)


def test_stats_one_sided_update_leaves_the_other_factor_alone():
    G = W.gaussian_block(70, 90, 0.1, DEV, 3, dtype=torch.bfloat16)
    L = spd(70, 3); R = spd(90, 4); R0 = R.clone()
    Lo, _ = oracle.stats_update(np64(G), np64(L), np64(R), 0.5)
    ast.stats_update([(G, L, None)], 0.5)
    torch.cuda.synchronize()
    assert relF(L, Lo) <= TOL_STATS and torch.equal(R, R0)


def test_stats_full_size_1024_block_lowrank_bf16():
    n = 1024
    G = W.lowrank_block(n, n, DEV, 0)
    L = torch.zeros(n, n, device=DEV); R = torch.zeros(n, n, device=DEV)
    ast.stats_update([(G, L, R)], 0.95)
    torch.cuda.synchronize()
    Lo, Ro = oracle.stats_update(np64(G), np.zeros((n, n)), np.zeros((n, n)), 0.95)
    assert relF(L, Lo) <= TOL_STATS and relF(R, Ro) <= TOL_STATS


def ulps(a: torch.Tensor, b: np.ndarray) -> np.ndarray:
    """distance in fp32 units in the last place between a GPU fp32 tensor and float64 values rounded to fp32"""
    ai = a.detach().cpu().contiguous().numpy().view(np.int32).astype(np.int64)
    bi = np.ascontiguousarray(b.astype(np.float32)).view(np.int32).astype(np.int64)
    ai = np.where(ai < 0, -(ai & 0x7fffffff), ai)
    bi = np.where(bi < 0, -(bi & 0x7fffffff), bi)
    return np.abs(ai - bi)


def test_stats_fp64_accumulation_is_the_float64_update_rounded_once():
    # acc = ACC_F64: exact products, fp64 sums and EMA, one rounding to fp32.  beta is handed to the
    # oracle as the fp32 number the C ABI carries (1 - beta is then exact in fp32 as well), so the
    # oracle's float64 result rounded to fp32 is what the call must return, up to the order of the
    # float64 additions (which can move a value that lies within 1e-16 of a rounding boundary).
    beta = float(np.float32(0.9))
    shapes = [(200, 328, torch.bfloat16), (1, 1, torch.float32), (3, 5, torch.bfloat16), (130, 257, torch.float32),
              (256, 1024, torch.bfloat16), (129, 127, torch.bfloat16), (384, 128, torch.float32)]
    items, refs = [], []
    for i, (m, n, dt) in enumerate(shapes):
        G = padded(m, n, 3 if i % 2 else 0, dt, fill=5.0)
        G.copy_(W.gaussian_block(m, n, 0.1, DEV, 12, i, dtype=dt))
        L = padded(m, m, 5); L.copy_(spd(m, 11, i))
        R = padded(n, n, 0); R.copy_(spd(n, 12, i))
        refs.append(oracle.stats_update(np64(G), np64(L), np64(R), beta))
        items.append((G, L, R, B.ACC_F64))
    # one block of the same call keeps fp32 accumulation
    G32 = W.gaussian_block(256, 128, 0.1, DEV, 13, dtype=torch.bfloat16)
    L32, R32 = spd(256, 14), spd(128, 15)
    ref32 = oracle.stats_update(np64(G32), np64(L32), np64(R32), beta)
    ast.stats_update(items + [(G32, L32, R32)], beta)
    torch.cuda.synchronize()
    for (G, L, R, _), (Lo, Ro) in zip(items, refs):
        for X, Xo in ((L, Lo), (R, Ro)):
            u = ulps(X, Xo)
            assert u.max() <= 1 and (u > 0).mean() <= 1e-4, (tuple(G.shape), int(u.max()), float((u > 0).mean()))
            assert torch.equal(X, X.T)
        assert torch.all(L._base[:, L.shape[1]:] == -777.0) and torch.all(G._base[:, G.shape[1]:] == 5.0)
    assert relF(L32, ref32[0]) <= TOL_STATS and relF(R32, ref32[1]) <= TOL_STATS


def test_stats_fp64_accumulation_keeps_an_ill_conditioned_statistic_above_minus_half_eps():
    # the 4096 stress workload in miniature (singular values over 8 decades, eps = 1e-8 lambda_max):
    # the statistics of one update from zero are positive semi-definite up to round-off, and the root
    # needs lambda_min > -eps / 2.  fp64 accumulation leaves the rounding of the stored fp32 numbers as
    # the only error (about 1.4e-9 lambda_max); the oracle then grades the root of that very matrix.
    n = 512
    beta = float(np.float32(0.95))
    U, V = W.haar(n, DEV, 301, dtype=torch.float64), W.haar(n, DEV, 302, dtype=torch.float64)
    G = ((U * W.logspaced_sigma(n, 8.0, DEV)) @ V.T).to(torch.bfloat16)
    L = torch.zeros(n, n, device=DEV); R = torch.zeros(n, n, device=DEV)
    ast.stats_update([(G, L, R, B.ACC_F64)], beta)
    torch.cuda.synchronize()
    Lo, Ro = oracle.stats_update(np64(G), np.zeros((n, n)), np.zeros((n, n)), beta)
    assert ulps(L, Lo).max() <= 1 and ulps(R, Ro).max() <= 1
    eps = float(np.float32(1e-8))
    Xo, lmax_o, status = oracle.inverse_root_batch([np64(L), np64(R)], eps)
    assert np.all(status == oracle.OK)                    # the oracle does not clamp: positive definite with eps
    for A in (L, R):
        lam = np.linalg.eigvalsh(np64(A))
        assert lam[0] > -0.5 * eps * lam[-1], lam[0] / lam[-1]
    Xs, info, iters, resid, lmax = run_roots([L, R], eps)
    assert np.all(info == B.INFO_OK)
    for i in range(2):
        assert relF(Xs[i], Xo[i]) <= TOL_ROOT, relF(Xs[i], Xo[i])


# =============================================================================== packed lower-tile storage

def packed_reference(full64: np.ndarray) -> np.ndarray:
    """Packed lower tiles written out on the host (test-side helper): tile (ti, tj), tj <= ti, at index
    ti (ti + 1) / 2 + tj, 128 x 128 row-major, zero padding."""
    n = full64.shape[0]
    T = (n + 127) // 128
    pad = np.zeros((T * 128, T * 128))
    pad[:n, :n] = full64
    out = np.zeros((T * (T + 1) // 2, 128, 128))
    for ti in range(T):
        for tj in range(ti + 1):
            out[ti * (ti + 1) // 2 + tj] = pad[ti * 128:(ti + 1) * 128, tj * 128:(tj + 1) * 128]
    return out.reshape(-1)


def test_packed_storage_pack_and_unpack_round_trip():
    sizes = [1, 127, 128, 129, 300, 512]
    fulls = [padded(n, n, 3) for n in sizes]
    for i, (n, F) in enumerate(zip(sizes, fulls)):
        F.copy_(spd(n, 20, i))
    packs = [torch.full((ast.packed_elems(n),), float("nan"), device=DEV) for n in sizes]
    assert ast.packed_elems(1024) == 36 * 128 * 128 and ast.packed_elems(129) == 3 * 128 * 128
    ast.sym_pack(list(zip(fulls, packs)))
    backs = [padded(n, n, 1) for n in sizes]
    ast.sym_unpack(list(zip(backs, packs)))
    torch.cuda.synchronize()
    for n, F, P, Bk in zip(sizes, fulls, packs, backs):
        assert np.array_equal(P.cpu().numpy().astype(np.float64), packed_reference(np.tril(np64(F)) + np.tril(np64(F), -1).T))
        assert torch.equal(Bk, F) and torch.all(Bk._base[:, n:] == -777.0)


def test_stats_update_on_packed_statistics_and_roots_from_them():
    # L and R kept in packed lower tiles: the update reads and writes only the stored tiles; the result
    # equals the full-storage update bit for bit (same kernels, same sums), and the inverse root reads
    # the packed statistics directly.  Whole-tile bf16 blocks (the guard-free kernel), a ragged bf16 block,
    # an fp32 block and an fp64-accumulated one (the guarded kernels).
    cases = [(256, 384, torch.bfloat16, B.ACC_F32), (512, 256, torch.bfloat16, B.ACC_F32), (200, 328, torch.bfloat16, B.ACC_F32),
             (130, 257, torch.float32, B.ACC_F32), (129, 300, torch.bfloat16, B.ACC_F64)]
    items_f, items_p, keep = [], [], []
    for i, (m, n, dt, acc) in enumerate(cases):
        G = W.gaussian_block(m, n, 0.1, DEV, 30, i, dtype=dt)
        L, R = spd(m, 31, i), spd(n, 32, i)
        Lp = torch.full((ast.packed_elems(m),), float("nan"), device=DEV)
        Rp = torch.full((ast.packed_elems(n),), float("nan"), device=DEV)
        ast.sym_pack([(L, Lp), (R, Rp)])
        items_f.append((G, L, R, acc))
        items_p.append((G, Lp, Rp, acc, B.LAYOUT_PACKED))
        keep.append((m, n, L, R, Lp, Rp))
    refs = [oracle.stats_update(np64(G), np64(L), np64(R), 0.9) for (G, L, R, _) in items_f]
    ast.stats_update(items_f, 0.9)
    ast.stats_update(items_p, 0.9)
    torch.cuda.synchronize()
    for (m, n, L, R, Lp, Rp), (Lo, Ro) in zip(keep, refs):
        assert relF(L, Lo) <= TOL_STATS and relF(R, Ro) <= TOL_STATS
        Lb, Rb = torch.empty_like(L), torch.empty_like(R)
        ast.sym_unpack([(Lb, Lp), (Rb, Rp)])
        torch.cuda.synchronize()
        assert torch.equal(Lb, L) and torch.equal(Rb, R), (m, n)
    # roots of the packed statistics against the oracle (fed the unpacked arrays) and against the full path
    As_p = [k[4] for k in keep] + [k[5] for k in keep]
    As_f = [k[2] for k in keep] + [k[3] for k in keep]
    Xp = [torch.full_like(A, float("nan")) for A in As_f]
    Xf = [torch.full_like(A, float("nan")) for A in As_f]
    info = torch.full((2 * len(As_f),), -1, dtype=torch.int32, device=DEV)
    lm = torch.zeros(2 * len(As_f), device=DEV)
    ast.inverse_root([(A, X, B.LAYOUT_PACKED) for A, X in zip(As_p, Xp)] + list(zip(As_f, Xf)), 1e-4, info=info, lambda_max=lm)
    torch.cuda.synchronize()
    assert torch.all(info == 0)
    k = len(As_f)
    for i, (A, X, Xfull) in enumerate(zip(As_f, Xp, Xf)):
        Xo, lmax_o, _ = oracle.inverse_root(np64(A), 1e-4)
        assert relF(X, Xo) <= TOL_ROOT and relF(Xfull, Xo) <= TOL_ROOT
        assert abs(float(lm[i]) - lmax_o) <= 1e-3 * lmax_o and abs(float(lm[k + i]) - lmax_o) <= 1e-3 * lmax_o
        assert relF(X, np64(Xfull)) <= 1e-4        # the two mat-vec kernels sum in different orders


# =============================================================================== a2 inverse roots

def test_root_single_block_config_absolute_and_relative_eps():
    n = 128
    L = torch.eye(n, device=DEV); R = torch.eye(n, device=DEV)
    for k in range(8):
        ast.stats_update([(W.gaussian_block(n, n, 0.01, DEV, 1, k), L, R)], 0.95)
    for A in (L, R):
        Xo, lmax_o, lam = oracle.inverse_root(np64(A), 1e-6)
        assert lam.max() / lam.min() < 1.05
        (X,), info, iters, resid, lmax = run_roots([A], 1e-6)
        assert info[0] == B.INFO_OK and 1 <= iters[0] <= 4
        # nearly flat spectrum (width ~1%): 128 eigenvalues within 1 % of each other
        assert abs(lmax[0] - lmax_o) <= 1e-4 * lmax_o
        assert relF(X, Xo) <= TOL_ROOT
        (Xa,), info, _, _, _ = run_roots([A], 1e-6 * lmax_o, relative=False)
        assert info[0] == B.INFO_OK and relF(Xa, Xo) <= 1e-5
        assert torch.equal(Xa, Xa.T)
        # default options: the iterations after the fp64 prefix run on split-fp16 products and the look-ahead
        # stop rule accepts a truncation error of 7e-4 per eigen-direction (bar: 2e-3)
        assert relF(X, Xo) <= 1e-3


@pytest.mark.parametrize("schedule", [1, 0])
@pytest.mark.parametrize("n", [200, 320])
def test_root_powerlaw_spectrum_ragged_sizes(n, schedule):
    A = powerlaw_factor(n, 11)
    Xo, lmax_o, lam = oracle.inverse_root(np64(A), 1e-6)
    for j in (0, -1, 40):       # fp32 only, automatic fp64 prefix, fp64 throughout
        (X,), info, iters, resid, lmax = run_roots([A], 1e-6, opts=ast.RootOpts(fp64_iters=j, schedule=schedule))
        assert info[0] == B.INFO_OK
        assert abs(lmax[0] - lmax_o) <= 1e-4 * lmax_o
        assert relF(X, Xo) <= TOL_ROOT, (j, relF(X, Xo))
        assert torch.equal(X, X.T)
    assert relF(X, Xo) <= 1e-5      # the fp64 run is limited only by the fp32 output and lambda_max


@pytest.mark.parametrize("schedule", [1, 0])
def test_root_of_lowrank_statistics_from_the_gpu_stats_kernel(schedule):
    # batch-of-64 workload in miniature: rank-32 + noise gradients, ~all eigenvalues on the eps floor
    n = 256
    G = W.lowrank_block(n, n, DEV, 7)
    L = torch.zeros(n, n, device=DEV); R = torch.zeros(n, n, device=DEV)
    ast.stats_update([(G, L, R)], 0.95)
    Xs, info, iters, resid, lmax = run_roots([L, R], 1e-6, opts=ast.RootOpts(schedule=schedule))
    for A, X, i in zip((L, R), Xs, range(2)):
        st, Xo, lmax_o, lam = oracle.inverse_root(np64(A), 1e-6, return_status=True)
        assert st == oracle.OK
        assert info[i] == B.INFO_OK and abs(lmax[i] - lmax_o) <= 1e-3 * lmax_o
        assert relF(X, Xo) <= TOL_ROOT, relF(X, Xo)


def test_root_ill_conditioned_logspaced_spectrum_eps_1e8():
    # 4096-block stress workload in miniature: singular values 1e0 .. 1e-8, eps = 1e-8 lambda_max
    n = 256
    A = logspaced_factor(n, 8.0, 5)
    st, Xo, lmax_o, lam = oracle.inverse_root(np64(A), 1e-8, return_status=True)
    assert st == oracle.OK and lam.min() > -0.5e-8 * lmax_o      # precondition of the workload
    (X,), info, iters, resid, lmax = run_roots([A], 1e-8)
    assert info[0] == B.INFO_OK
    assert relF(X, Xo) <= TOL_ROOT, relF(X, Xo)
    assert 9 <= iters[0] <= 14                      # interval-adapted coefficients
    # classical Newton coefficients need about twice as many iterations (and a longer fp64 prefix)
    (Xc,), info, iters_c, _, _ = run_roots([A], 1e-8, opts=ast.RootOpts(schedule=0))
    assert info[0] == B.INFO_OK and relF(Xc, Xo) <= TOL_ROOT
    assert 20 <= iters_c[0] <= 30


def test_root_fp64_iterations_on_the_int8_cores_against_the_fp64_cores_and_the_oracle():
    # The products of the fp64 iterations run on the int8 matrix cores (diagonal + 7-bit slices) where a
    # device-side estimate allows it, else on the fp64 cores.  Spectra and structures on both sides of
    # that decision: delocalised eigenvectors (small off-diagonal entries: 4 slices pass), an
    # equicorrelated matrix and a block-diagonal one with localised eigenvectors (off-diagonal entries
    # of the size of the diagonal: more slices, or the fp64 cores), a diagonal matrix (empty slices),
    # ragged sizes that are no multiple of the 32-wide slice blocks.
    n = 300
    ones = torch.ones(n, n, device=DEV, dtype=torch.float64)
    equi = 0.02 * (0.1 * torch.eye(n, device=DEV, dtype=torch.float64) + 0.9 * ones / n * 30)
    blk = torch.zeros(n, n, device=DEV, dtype=torch.float64)
    d = 0.05 * W.logspaced_sigma(n, 5.0, DEV).double() ** 2
    for i in range(0, n - 1, 2):                       # 2 x 2 blocks [[a, b], [b, a]]: eigenvectors (1, +-1)
        a_, b_ = 0.5 * (d[i] + d[i + 1]), 0.5 * (d[i] - d[i + 1])
        blk[i, i] = blk[i + 1, i + 1] = a_; blk[i, i + 1] = blk[i + 1, i] = b_
    cases = {"power law": powerlaw_factor(n, 21), "log-spaced": logspaced_factor(173, 6.0, 22),
             "equicorrelated": equi.float().contiguous(), "2x2 blocks": blk.float().contiguous(),
             "diagonal": torch.diag(d.float()).contiguous(), "small": powerlaw_factor(45, 23)}
    for name, A in cases.items():
        st, Xo, lmax_o, lam = oracle.inverse_root(np64(A), 1e-6, return_status=True)
        assert st == oracle.OK, name
        res = {}
        for ns in (-1, 0, 4):                           # library rule (up to 5 slices), fp64 cores only, 4 slices at most
            (X,), info, iters, resid, lmax = run_roots([A], 1e-6, opts=ast.RootOpts(int8_slices=ns))
            assert info[0] == B.INFO_OK, (name, ns)
            assert relF(X, Xo) <= TOL_ROOT, (name, ns, relF(X, Xo))
            assert torch.equal(X, X.T)
            res[ns] = (np64(X), int(iters[0]))
        assert res[-1][1] == res[0][1] == res[4][1], name   # the schedule does not depend on where the products run
        # the int8 path reproduces the fp64-core result far inside the tolerance
        assert relF(res[-1][0], res[0][0]) <= 2.5e-4, (name, relF(res[-1][0], res[0][0]))
        assert relF(res[4][0], res[0][0]) <= 2.5e-4, (name, relF(res[4][0], res[0][0]))
    # a factor longer than the rows the slicing kernel parks in LDS (2048): rows are read twice there;
    # 65 blocks of 32 k (an odd count), a ragged last tile
    # (too large for the oracle's Jacobi sweeps, minutes at this size: graded against the definition
    # V (lambda + eps)^(-1/4) V^T written out with a float64 eigendecomposition, and against the
    # fp64-core path)
    A = powerlaw_factor(2080, 24)
    w, V = torch.linalg.eigh(A.double())
    Xdef = (V * (w + 1e-6 * w[-1]) ** -0.25) @ V.T
    got = {}
    for ns in (-1, 0):
        (X,), info, iters, resid, lmax = run_roots([A], 1e-6, opts=ast.RootOpts(int8_slices=ns))
        assert info[0] == B.INFO_OK
        got[ns] = X.double()
        err = float((got[ns] - Xdef).norm() / Xdef.norm())
        assert err <= TOL_ROOT, (ns, err)
    assert float((got[-1] - got[0]).norm() / got[0].norm()) <= 2.5e-4
    # a batch: every factor takes its own decision
    As = list(cases.values())
    Xs, info, iters, resid, lmax = run_roots(As, 1e-6)
    for A, X in zip(As, Xs):
        Xo, _, _ = oracle.inverse_root(np64(A), 1e-6)
        assert relF(X, Xo) <= TOL_ROOT


def test_root_int8_decision_over_spectra_structures_and_prefix_lengths():
    # The device-side decision of the int8 path (4 slices, 5 slices or the fp64 cores, per factor and
    # product) against the fp64-core path: spectra with wide and narrow gaps, eigenvectors spread over
    # all coordinates or confined to 2 and 4 of them (off-diagonal entries as large as the diagonal),
    # and eps = 1e-8, where the fp64 prefix is four iterations long and twelve products share the error
    # budget.  Reference: the definition V (lambda + eps)^(-1/4) V^T with a float64 eigendecomposition
    # (the oracle's Jacobi sweeps would take minutes for this many matrices).
    def spec_matrix(n, lam, width):
        if width == 0:
            U = W.haar(n, DEV, 31, dtype=torch.float64)
            A = (U * lam) @ U.T
        else:
            A = torch.zeros(n, n, device=DEV, dtype=torch.float64)
            perm = torch.randperm(n, device=DEV, generator=torch.Generator(DEV).manual_seed(5))
            lp = lam[perm]
            for b in range(0, n, width):
                w = min(width, n - b)
                U = W.haar(w, DEV, 40 + b, dtype=torch.float64)
                A[b:b + w, b:b + w] = (U * lp[b:b + w]) @ U.T
        return (0.5 * (A + A.T)).float().contiguous()
    worst = 0.0
    for n in (96, 512):
        i = torch.arange(1, n + 1, device=DEV, dtype=torch.float64)
        spectra = {"power law": 0.05 / i ** 2, "8 decades": 0.05 * 10 ** (-8 * (i - 1) / (n - 1)),
                   "two levels": torch.where(i <= n // 2, 1.0, 1e-5) * 0.05}
        for sname, lam in spectra.items():
            for width in (0, 4, 2):
                A = spec_matrix(n, lam, width)
                w, V = torch.linalg.eigh(A.double())
                for eps in (1e-6, 1e-8):
                    Xdef = (V * (w + eps * w[-1]).clamp_min(1e-300) ** -0.25) @ V.T
                    got = {}
                    for ns in (-1, 0):
                        (X,), info, iters, resid, lmax = run_roots([A], eps, opts=ast.RootOpts(int8_slices=ns))
                        assert info[0] == B.INFO_OK, (n, sname, width, eps, ns)
                        got[ns] = X.double()
                        err = float((got[ns] - Xdef).norm() / Xdef.norm())
                        assert err <= TOL_ROOT, (n, sname, width, eps, ns, err)
                    dev = float((got[-1] - got[0]).norm() / got[0].norm())
                    worst = max(worst, dev)
                    assert dev <= 2.5e-4, (n, sname, width, eps, dev)
    print("int8 path against the fp64-core path, worst relF", worst)


def newton_count(a: float, n: int, stop: float = 1e-2, p: int = 4) -> int:
    """Scalar model of the coupled iteration on the smallest eigenvalue a of M_0."""
    mu, k = a, 0
    while math.sqrt(n) * abs(1 - mu) >= stop and k < 100:
        mu = ((p + 1 - mu) / p) ** p * mu
        k += 1
    return k + 1


def test_root_iteration_counts_follow_the_scalar_recurrence():
    n = 192
    counts, adapted = {}, {}
    for kappa in (1e2, 1e4, 1e6):
        U = W.haar(n, DEV, 21, dtype=torch.float64)
        lam = torch.logspace(0, -math.log10(kappa), n, device=DEV, dtype=torch.float64)
        A = ((U * lam) @ U.T)
        A = (0.5 * (A + A.T)).float().contiguous()
        (X,), info, iters, _, _ = run_roots([A], 1e-12, opts=ast.RootOpts(schedule=0))
        assert info[0] == B.INFO_OK
        counts[kappa] = int(iters[0])
        # the adapted schedule is built for the interval [~0.5 eps s, 1]; pass eps = lambda_min so
        # that the interval matches the spectrum
        (X,), info, iters, _, _ = run_roots([A], 1.0 / kappa)
        assert info[0] == B.INFO_OK
        adapted[kappa] = int(iters[0])
        # all n eigenvalues at the bottom is the worst case of the model; one at the bottom the best
        assert newton_count(1 / (1.01 * kappa), 1) - 1 <= counts[kappa] <= newton_count(1 / (1.01 * kappa), n) + 1
    assert counts[1e2] < counts[1e4] < counts[1e6]
    assert adapted[1e4] <= 0.7 * counts[1e4] and adapted[1e6] <= 0.6 * counts[1e6]


def test_root_inverse_square_root():
    A = powerlaw_factor(160, 31)
    Xo, _, _ = oracle.inverse_root(np64(A), 1e-4, p=2)
    (X,), info, _, _, _ = run_roots([A], 1e-4, root=2)
    assert info[0] == B.INFO_OK and relF(X, Xo) <= TOL_ROOT


def test_root_mixed_batch_multiple_passes_and_padded_outputs():
    sizes = [64, 300, 1, 129, 200, 17]
    As = [powerlaw_factor(n, 40 + i) for i, n in enumerate(sizes)]
    refs = [oracle.inverse_root(np64(A), 1e-5)[0] for A in As]
    full, mn = ast.inverse_root_workspace_bytes(list(zip(As, As)))
    assert mn < full
    for nbytes in (full, mn + 4096):          # one pass, then as many passes as the smallest workspace forces
        ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
        Xs = []
        for A in As:
            Xs.append(padded(A.shape[0], A.shape[0], 4))
        info = torch.full((len(As),), -1, dtype=torch.int32, device=DEV)
        ast.inverse_root(list(zip(As, Xs)), [1e-5] * len(As), info=info, ws=ws)
        torch.cuda.synchronize()
        assert torch.all(info == 0)
        for X, Xo in zip(Xs, refs):
            assert relF(X, Xo) <= TOL_ROOT
            assert torch.all(X._base[:, X.shape[1]:] == -777.0)
    with pytest.raises(ast.AsteriaError) as e:
        ast.inverse_root(list(zip(As, Xs)), 1e-5, ws=torch.empty(mn - 4096, dtype=torch.uint8, device=DEV))
    assert e.value.status == B.WORKSPACE_TOO_SMALL


def test_root_spectra_that_stress_the_stop_rules():
    # spectra for which a stop test based on the interval predicted for M could stop too early or the
    # adapted coefficients could misbehave: one dominant eigenvalue over a floor far below eps; two
    # tight clusters three decades apart; a flat spectrum (kappa = 1); a gap right at eps
    n = 256
    U = W.haar(n, DEV, 60, dtype=torch.float64)
    def build(lam):
        A = (U * lam) @ U.T
        return (0.5 * (A + A.T)).float().contiguous()
    one = torch.ones(n, device=DEV, dtype=torch.float64)
    spectra = {
        "spike": torch.cat([torch.tensor([1.0], device=DEV, dtype=torch.float64), 1e-9 * one[1:]]),
        "clusters": torch.cat([1.0 + 1e-3 * torch.arange(n // 2, device=DEV, dtype=torch.float64) / n,
                               1e-3 * (1.0 + 1e-3 * torch.arange(n // 2, device=DEV, dtype=torch.float64) / n)]),
        "flat": 0.37 * one,
        "gap at eps": torch.cat([torch.linspace(1.0, 0.1, n // 2, device=DEV, dtype=torch.float64), 1e-6 * one[: n // 2]]),
    }
    As = [build(lam) for lam in spectra.values()]
    for schedule in (1, 0):
        Xs, info, iters, resid, _ = run_roots(As, 1e-6, opts=ast.RootOpts(schedule=schedule))
        Xo, _, status = oracle.inverse_root_batch([np64(A) for A in As], 1e-6)
        assert np.all(status == oracle.OK) and np.all(info == B.INFO_OK), (schedule, info)
        errs = {k: relF(X, Xo[i]) for i, (k, X) in enumerate(zip(spectra, Xs))}
        print("stop-rule stress, schedule", schedule, "iters", iters, errs)
        assert max(errs.values()) <= TOL_ROOT, (schedule, errs)


def test_root_failure_reporting_is_per_factor():
    good = powerlaw_factor(96, 50)
    bad = good.clone()
    bad -= 0.5 * torch.eye(96, device=DEV) * good.diagonal().max()      # strongly indefinite
    Xo, _, _ = oracle.inverse_root(np64(good), 1e-6)
    st, _, _, _ = oracle.inverse_root(np64(bad), 1e-6, return_status=True)
    assert st == oracle.NOT_PD
    Xs, info, iters, resid, lmax = run_roots([good, bad, good], 1e-6)
    assert info[0] == B.INFO_OK and info[2] == B.INFO_OK and info[1] in (B.INFO_NOT_PD, B.INFO_NOT_CONVERGED)
    assert relF(Xs[0], Xo) <= TOL_ROOT and torch.equal(Xs[0], Xs[2])
    # an exhausted iteration budget is reported, not hidden
    _, info, iters, _, _ = run_roots([good], 1e-6, opts=ast.RootOpts(max_iters=1))
    assert info[0] == B.INFO_NOT_CONVERGED and iters[0] == 1
    # a zero matrix has no relative regularisation: not positive definite
    _, info, _, _, _ = run_roots([torch.zeros(8, 8, device=DEV)], 1e-6)
    assert info[0] == B.INFO_NOT_PD
    # ... but with an absolute eps it is eps^-1/4 I
    (X,), info, _, _, _ = run_roots([torch.zeros(8, 8, device=DEV)], 1e-4, relative=False)
    assert info[0] == B.INFO_OK and relF(X, 10.0 * np.eye(8)) <= 1e-5


def test_root_full_size_1024_factors_against_the_oracle():
    # two factors at the size of the headline workload (oracle: ~1.5 min per factor, run in parallel)
    n = 1024
    bank = W.TemplateBank(DEV)
    Gp = W.powerlaw_blocks([(n, n)], DEV, bank=bank)[0]
    Gl = W.lowrank_block(n, n, DEV, 1)
    Ls = [torch.zeros(n, n, device=DEV) for _ in range(2)]
    ast.stats_update([(Gp, Ls[0], None), (Gl, Ls[1], None)], 0.95)
    Xs, info, iters, resid, lmax = run_roots(Ls, 1e-6)
    Xo, lmax_o, status = oracle.inverse_root_batch([np64(A) for A in Ls], 1e-6)
    assert np.all(status == oracle.OK) and np.all(info == B.INFO_OK)
    for i in range(2):
        assert abs(lmax[i] - lmax_o[i]) <= 1e-3 * lmax_o[i]
        assert relF(Xs[i], Xo[i]) <= TOL_ROOT, (i, relF(Xs[i], Xo[i]))
    print("iters", iters, "relF", [relF(Xs[i], Xo[i]) for i in range(2)])


# =============================================================================== a3 precondition

def test_precondition_ragged_batch_fp32_and_bf16_outputs():
    shapes = [(128, 128, torch.float32, torch.float32), (200, 328, torch.bfloat16, torch.float32),
              (5, 3, torch.float32, torch.float32), (257, 130, torch.bfloat16, torch.bfloat16), (1, 1, torch.bfloat16, torch.float32)]
    items, refs = [], []
    for i, (m, n, gdt, pdt) in enumerate(shapes):
        G = W.gaussian_block(m, n, 0.01, DEV, 5, i, dtype=gdt)
        XL, XR = spd(m, 5, i), spd(n, 6, i)
        P = padded(m, n, 2, pdt)
        refs.append(oracle.precondition(np64(XL), np64(G), np64(XR)))
        items.append((XL, G, XR, P))
    ast.precondition(items)
    torch.cuda.synchronize()
    for (XL, G, XR, P), Po, (_, _, gdt, pdt) in zip(items, refs, shapes):
        # fp32 gradients run on the fp32 matrix cores; bf16 gradients on the bf16 cores with the
        # roots split into two bf16 terms (~16 bits); a bf16 store rounds to 8 bits
        tol = TOL_PRECOND if pdt == torch.bfloat16 else (1e-4 if gdt == torch.bfloat16 else 1e-5)
        print("precondition", tuple(G.shape), gdt, pdt, relF(P, Po))
        assert relF(P, Po) <= tol, relF(P, Po)
        assert torch.all(P._base[:, P.shape[1]:] == -777.0)


def test_precondition_whole_tile_blocks_mixed_with_ragged_ones():
    # blocks whose shapes fill whole 256 x 256 tiles take another kernel for the second product than
    # the ragged block in the same call
    shapes = [(256, 512, torch.bfloat16), (200, 328, torch.bfloat16), (512, 256, torch.bfloat16), (256, 256, torch.bfloat16)]
    items, refs = [], []
    for i, (m, n, gdt) in enumerate(shapes):
        G = W.gaussian_block(m, n, 0.01, DEV, 7, i, dtype=gdt)
        XL, XR = spd(m, 8, i), spd(n, 9, i)
        P = padded(m, n, 4 if i % 2 == 0 else 1, torch.float32)   # 16-byte rows, and rows that are not
        refs.append(oracle.precondition(np64(XL), np64(G), np64(XR)))
        items.append((XL, G, XR, P))
    ast.precondition(items)
    torch.cuda.synchronize()
    for (XL, G, XR, P), Po in zip(items, refs):
        print("precondition whole tiles", tuple(G.shape), relF(P, Po))
        assert relF(P, Po) <= 1e-4, relF(P, Po)
        assert torch.all(P._base[:, P.shape[1]:] == -777.0)


def test_precondition_full_size_1024_with_gpu_roots():
    n = 1024
    G = W.powerlaw_blocks([(n, n)], DEV)[0]
    L = torch.zeros(n, n, device=DEV); R = torch.zeros(n, n, device=DEV)
    ast.stats_update([(G, L, R)], 0.95)
    (XL, XR), info, _, _, _ = run_roots([L, R], 1e-6)
    assert np.all(info == 0)
    P = torch.empty(n, n, device=DEV)
    ast.precondition([(XL, G, XR, P)])
    torch.cuda.synchronize()
    Po = oracle.precondition(np64(XL), np64(G), np64(XR))
    print("precondition 1024 relF", relF(P, Po))
    assert relF(P, Po) <= 1e-4      # split-bf16 roots; the stated bar is 1e-2


def test_end_to_end_single_block_config_against_the_float64_pipeline():
    n = 128
    L = torch.eye(n, device=DEV); R = torch.eye(n, device=DEV)
    Lo, Ro = np.eye(n), np.eye(n)
    for k in range(8):
        G = W.gaussian_block(n, n, 0.01, DEV, 1, k)
        ast.stats_update([(G, L, R)], 0.95)
        Lo, Ro = oracle.stats_update(np64(G), Lo, Ro, 0.95)
    (XL, XR), info, _, _, _ = run_roots([L, R], 1e-6)
    P = torch.empty(n, n, device=DEV)
    ast.precondition([(XL, G, XR, P)])
    torch.cuda.synchronize()
    XLo, _, _ = oracle.inverse_root(Lo, 1e-6)
    XRo, _, _ = oracle.inverse_root(Ro, 1e-6)
    Po = oracle.precondition(XLo, np64(G), XRo)
    assert relF(XL, XLo) <= TOL_ROOT and relF(XR, XRo) <= TOL_ROOT and relF(P, Po) <= TOL_PRECOND
    assert abs(float(XL.diagonal().mean()) - 0.95 ** -2) < 0.01


def test_full_model_batch_in_the_timed_launch_configuration_sampled_against_the_oracle():
    # the headline workload exactly as the benchmark launches it: all 1184 blocks / 2368 factors of
    # the 1.1B model in one call per stage on one shared workspace; a sample of blocks that covers
    # every block shape and both ends of the batch is checked stage by stage against the oracle
    shapes = W.block_shapes(W.llama_1b_matrices(), 1024)
    nb = len(shapes)
    Gs = W.powerlaw_blocks(shapes, DEV)
    Ls = [torch.zeros(m, m, device=DEV) for m, n in shapes]
    Rs = [torch.zeros(n, n, device=DEV) for m, n in shapes]
    XLs = [torch.empty(m, m, device=DEV) for m, n in shapes]
    XRs = [torch.empty(n, n, device=DEV) for m, n in shapes]
    Ps = [torch.empty(m, n, device=DEV) for m, n in shapes]
    blocks = ast.Blocks(list(zip(Gs, Ls, Rs)))
    factors = ast.Factors([(L, X) for L, X in zip(Ls, XLs)] + [(R, X) for R, X in zip(Rs, XRs)])
    pblocks = ast.PBlocks(list(zip(XLs, Gs, XRs, Ps)))
    full, mn = ast.inverse_root_workspace_bytes(factors, None)
    ws_bytes = int(max(min(full, 128 * 2**30), mn,       # as the benchmark: all 2368 factors in one pass (107 GiB) ast.precondition_workspace_bytes(pblocks),
                       ast.stats_update_workspace_bytes(blocks)))
    assert ws_bytes >= full, "the timed configuration is a single pass"
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    info = torch.full((2 * nb,), -1, dtype=torch.int32, device=DEV)
    ast.stats_update(blocks, 0.95, ws=ws)
    ast.inverse_root(factors, 1e-6, relative=True, root=4, info=info, ws=ws)
    ast.precondition(pblocks, ws=ws)
    torch.cuda.synchronize()
    assert np.all(info.cpu().numpy() == B.INFO_OK)

    # first and last block of every shape; the oracle's eigensolver sets the cost (about 1.5 min for
    # n = 1024), so roots are checked on the small side of each sampled block, plus one 1024 factor
    # from each end of the batch
    sample = {}
    for i, sh in enumerate(shapes):
        sample.setdefault(sh, [i, i])[1] = i
    picks = sorted({i for pair in sample.values() for i in pair})
    root_jobs = []          # (GPU statistic, GPU root)
    for i in picks:
        m, n = shapes[i]
        Lo, Ro = oracle.stats_update(np64(Gs[i]), np.zeros((m, m)), np.zeros((n, n)), 0.95)
        assert relF(Ls[i], Lo) <= TOL_STATS and relF(Rs[i], Ro) <= TOL_STATS, (i, shapes[i])
        Po = oracle.precondition(np64(XLs[i]), np64(Gs[i]), np64(XRs[i]))
        assert relF(Ps[i], Po) <= 1e-4, (i, shapes[i], relF(Ps[i], Po))
        if min(m, n) < 1024:
            root_jobs.append((Ls[i], XLs[i]) if m <= n else (Rs[i], XRs[i]))
    root_jobs.append((Ls[picks[0]], XLs[picks[0]]))
    root_jobs.append((Rs[picks[-1]], XRs[picks[-1]]))
    Xo, _, status = oracle.inverse_root_batch([np64(A) for A, _ in root_jobs], 1e-6)
    assert np.all(status == oracle.OK)
    errs = [relF(X, Xo[j]) for j, (_, X) in enumerate(root_jobs)]
    print("full model: sampled blocks", [(i, shapes[i]) for i in picks], "root relF", errs)
    assert max(errs) <= TOL_ROOT, errs


# =============================================================================== a4 SOAP refresh

@pytest.mark.parametrize("n", [64, 200, 320])
def test_soap_refresh_invariants_and_leading_columns(n):
    A = powerlaw_factor(n, 60)
    Q0 = W.haar(n, DEV, 61)
    for _ in range(3):                                  # warm the basis from a random start
        ast.soap_refresh([(A, Q0)])
    Qin = Q0.clone()
    info = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    ast.soap_refresh([(A, Q0)], info=info)
    torch.cuda.synchronize()
    assert info.item() == 0
    Q = np64(Q0)
    Z = np64(A) @ np64(Qin)
    assert np.linalg.norm(Q.T @ Q - np.eye(n)) / math.sqrt(n) <= 1e-5
    Rm = Q.T @ Z
    assert np.linalg.norm(np.tril(Rm, -1)) <= 1e-5 * np.linalg.norm(Z)       # Q^T Z is upper triangular
    assert np.linalg.norm(Q @ np.triu(Rm) - Z) <= 1e-5 * np.linalg.norm(Z)   # backward error
    assert np.all(np.diag(Rm) >= -1e-7 * np.abs(Rm).max())
    Qo, Ro = oracle.soap_refresh(np64(A), np64(Qin))
    lead = min(32, n)
    assert np.all(np.abs(np.sum(Q[:, :lead] * Qo[:, :lead], axis=0)) >= 0.999)
    assert np.all(np.sum(Q[:, :lead] * Qo[:, :lead], axis=0) > 0)          # same sign convention


@pytest.mark.parametrize("n", [31, 129, 173, 257])
def test_soap_refresh_odd_sizes_in_a_padded_buffer(n):
    # Q lives in a buffer with an odd leading dimension (rows not 16-byte aligned): the split-fp16
    # products read and the panel transposes write the caller's Q through their guarded paths, and the
    # padding columns stay untouched
    G = W.gaussian_block(n, 3 * n, 1.0, DEV, 80 + n)
    A = (G @ G.T / (3 * n)).contiguous()
    buf = torch.full((n, n + 3), 7.0, device=DEV)
    buf[:, :n] = W.haar(n, DEV, 81 + n)
    Q = buf[:, :n]
    Qin = Q.clone()
    info = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    ast.soap_refresh([(A, Q)], info=info)
    torch.cuda.synchronize()
    assert info.item() == 0 and bool((buf[:, n:] == 7.0).all())
    q = np64(Q.contiguous()); Z = np64(A) @ np64(Qin.contiguous())
    assert np.linalg.norm(q.T @ q - np.eye(n)) / math.sqrt(n) <= 1e-5
    Rm = q.T @ Z
    assert np.linalg.norm(np.tril(Rm, -1)) <= 1e-5 * np.linalg.norm(Z)
    assert np.linalg.norm(q @ np.triu(Rm) - Z) <= 1e-5 * np.linalg.norm(Z)
    Qo, Ro = oracle.soap_refresh(np64(A), np64(Qin.contiguous()))
    lead = min(16, n)
    assert np.all(np.sum(q[:, :lead] * Qo[:, :lead], axis=0) >= 0.999)


def test_soap_refresh_fixed_points_and_batch():
    d = torch.linspace(3.0, 0.5, 40, device=DEV)
    A1 = torch.diag(d).contiguous(); Q1 = torch.eye(40, device=DEV)
    n = 96
    Qs = W.haar(n, DEV, 70, dtype=torch.float64)
    lam = torch.linspace(2.0, 0.1, n, device=DEV, dtype=torch.float64)
    A2 = ((Qs * lam) @ Qs.T)
    A2 = (0.5 * (A2 + A2.T)).float().contiguous(); Q2 = Qs.float().contiguous()
    Q2in = Q2.clone()
    ast.soap_refresh([(A1, Q1), (A2, Q2)])
    torch.cuda.synchronize()
    assert relF(Q1, np.eye(40)) <= 1e-6
    assert relF(Q2, Q2in) <= 1e-4


def test_soap_refresh_on_caller_streams_equals_the_single_stream_call():
    # the factors of a call dealt to groups on auxiliary streams of the caller: same kernels per factor,
    # so the result is bit-identical to the call that stays on one stream; the caller's stream waits for
    # the auxiliary ones (the comparison below is enqueued on it right after the call)
    sizes = [300, 129, 512, 64, 200, 257, 96]
    As = [powerlaw_factor(n, 70 + i) for i, n in enumerate(sizes)]
    Q0 = [W.haar(n, DEV, 71 + i) for i, n in enumerate(sizes)]
    ref = [q.clone() for q in Q0]
    info = torch.full((len(sizes),), -1, dtype=torch.int32, device=DEV)
    ast.soap_refresh(list(zip(As, ref)), info=info)
    torch.cuda.synchronize()
    assert torch.all(info == 0)
    for n_aux in (1, 2, 3):
        aux = [torch.cuda.Stream() for _ in range(n_aux)]
        Qs = [q.clone() for q in Q0]
        info.fill_(-1)
        ast.soap_refresh(list(zip(As, Qs)), info=info, aux_streams=aux)
        same = [torch.equal(a, b) for a, b in zip(Qs, ref)]        # on the caller's stream, no host wait in between
        torch.cuda.synchronize()
        assert all(same) and torch.all(info == 0), (n_aux, same)


def spectrum_factor(n, lam, *key):
    U = W.haar(n, DEV, *key, dtype=torch.float64)
    A = (U * lam) @ U.T
    return (0.5 * (A + A.T)).float().contiguous(), U.float().contiguous()


def test_soap_refresh_leaves_the_transposed_basis_in_a_buffer_of_the_caller():
    """With buffers for Q^T the refresh reads its operand from them instead of transposing Q in place and
    leaves the new Q^T there: same values through the same products, so Q is bit-identical to the plain
    call, Q^T is its exact transpose, and a second refresh that is told the buffers are valid agrees too."""
    ns = [200, 257, 64, 320]
    As = [powerlaw_factor(n, 120 + i) for i, n in enumerate(ns)]
    Q0 = [W.haar(n, DEV, 130 + i) for i, n in enumerate(ns)]
    ref = [q.clone() for q in Q0]
    ast.soap_refresh(list(zip(As, ref)))
    ast.soap_refresh(list(zip(As, ref)))
    Qs = [q.clone() for q in Q0]
    Qt = [padded(n, n, 4) if i % 2 else torch.full((n, n), float("nan"), device=DEV) for i, n in enumerate(ns)]
    Qt[2] = None                                                     # a factor without such a buffer
    info = torch.full((len(ns),), -1, dtype=torch.int32, device=DEV)
    ast.soap_refresh(list(zip(As, Qs)), info=info, qt=Qt)                      # buffers not filled yet
    ast.soap_refresh(list(zip(As, Qs)), info=info, qt=Qt, qt_valid=True)       # ... now they are
    torch.cuda.synchronize()
    assert np.all(info.cpu().numpy() == B.INFO_OK)
    for q, r, t in zip(Qs, ref, Qt):
        assert torch.equal(q, r)
        if t is not None:
            assert torch.equal(t, q.T)
    # sorted, from the identity, two rounds, on two streams: the same against the call without buffers
    ref = [torch.empty_like(q) for q in Q0]
    aux = [torch.cuda.Stream(), torch.cuda.Stream()]
    ast.soap_refresh(list(zip(As, ref)), sort=True, from_identity=True, rounds=2, aux_streams=aux)
    Qs = [torch.empty_like(q) for q in Q0]
    Qt = [torch.full((n, n), float("nan"), device=DEV) for n in ns]
    ast.soap_refresh(list(zip(As, Qs)), sort=True, from_identity=True, rounds=2, aux_streams=aux, qt=Qt)
    torch.cuda.synchronize()
    for q, r, t in zip(Qs, ref, Qt):
        assert torch.equal(q, r) and torch.equal(t, q.T)


def test_soap_refresh_in_several_passes_through_a_small_workspace():
    """A workspace that holds the largest factor only: the call works through the batch in passes (with
    two stream groups and kept transposes) and must return what the one-pass call returns."""
    ns = [257, 64, 200, 130, 31]
    As = [powerlaw_factor(n, 140 + i) for i, n in enumerate(ns)]
    Q0 = [W.haar(n, DEV, 150 + i) for i, n in enumerate(ns)]
    ref = [q.clone() for q in Q0]
    ast.soap_refresh(list(zip(As, ref)), sort=True)
    full, smallest = ast.soap_refresh_workspace_bytes(list(zip(As, Q0)))
    assert smallest < full
    ws = torch.empty(smallest, dtype=torch.uint8, device=DEV)
    aux = [torch.cuda.Stream(), torch.cuda.Stream()]
    Qs = [q.clone() for q in Q0]
    Qt = [torch.full((n, n), float("nan"), device=DEV) for n in ns]
    info = torch.full((len(ns),), -1, dtype=torch.int32, device=DEV)
    ast.soap_refresh(list(zip(As, Qs)), info=info, ws=ws, sort=True, aux_streams=aux, qt=Qt)
    torch.cuda.synchronize()
    assert np.all(info.cpu().numpy() == B.INFO_OK)
    for q, r, t in zip(Qs, ref, Qt):
        assert torch.equal(q, r) and torch.equal(t, q.T)


def test_soap_refresh_with_columns_ordered_by_estimated_eigenvalue():
    # sort = 1: the columns of the basis take the order of decreasing q^T A q before the power iteration
    # (the order SOAP keeps its basis in).  Spectra with well separated estimates, so that the order is
    # unique and the fp32 / fp64 estimates cannot disagree; the order is reported per factor.
    sizes = [200, 129, 320]
    As, Q0s = [], []
    for i, n in enumerate(sizes):
        lam = torch.logspace(0, -2, n, device=DEV, dtype=torch.float64)      # neighbours 2 - 4 % apart
        A, U = spectrum_factor(n, lam, 400 + i)
        g = torch.Generator(device=DEV).manual_seed(7 + i)
        shuffle = torch.randperm(n, device=DEV, generator=g)
        Q0 = U[:, shuffle].contiguous() if i < 2 else W.haar(n, DEV, 410 + i)    # shuffled eigenvectors, and a generic basis
        As.append(A); Q0s.append(Q0)
    Qs = [q.clone() for q in Q0s]
    perm = torch.full((sum(sizes),), -1, dtype=torch.int32, device=DEV)
    info = torch.full((len(sizes),), -1, dtype=torch.int32, device=DEV)
    ast.soap_refresh(list(zip(As, Qs)), info=info, sort=True, perm=perm)
    torch.cuda.synchronize()
    assert torch.all(info == 0)
    off = 0
    for n, A, Q0, Q in zip(sizes, As, Q0s, Qs):
        p_gpu = perm[off:off + n].cpu().numpy().astype(np.int64); off += n
        Qsorted, p_or, est = oracle.soap_sort(np64(A), np64(Q0))
        assert sorted(p_gpu.tolist()) == list(range(n))
        # The order is unique where the estimates are apart; columns whose estimates agree to fp32
        # round-off (a generic basis has many: every estimate is near tr A / n) may come in either
        # order.  So: the same column as the oracle's wherever that column's estimate is isolated, and
        # everywhere estimates that do not increase by more than the round-off of the fp32 data.
        tol = 2e-6 * np.abs(est).max()
        e_gpu, e_or = est[p_gpu], est[p_or]
        assert np.all(np.diff(e_gpu) <= tol)
        assert np.all(np.abs(e_gpu - e_or) <= tol)
        isolated = np.ones(n, dtype=bool)
        isolated[1:] &= -np.diff(e_or) > 2 * tol
        isolated[:-1] &= -np.diff(e_or) > 2 * tol
        assert np.array_equal(p_gpu[isolated], p_or[isolated])
        if Q0 is Q0s[0] or Q0 is Q0s[1]:
            assert isolated.all() and np.array_equal(p_gpu, p_or)      # shuffled eigenvectors: estimates = eigenvalues, all apart
        # the refresh itself, stage-wise: the oracle refreshes the basis in the order the GPU chose
        Qo, Ro = oracle.soap_refresh(np64(A), np64(Q0)[:, p_gpu])
        q = np64(Q)
        Z = np64(A) @ np64(Q0)[:, p_gpu]
        assert np.linalg.norm(q.T @ q - np.eye(n)) / math.sqrt(n) <= 1e-5
        Rm = q.T @ Z
        assert np.linalg.norm(np.tril(Rm, -1)) <= 1e-5 * np.linalg.norm(Z)
        assert np.linalg.norm(q @ np.triu(Rm) - Z) <= 1e-5 * np.linalg.norm(Z)
        lead = 32
        assert np.all(np.sum(q[:, :lead] * Qo[:, :lead], axis=0) >= 0.999)


def test_soap_refresh_from_the_identity_in_several_sorted_rounds_approaches_the_eigenbasis():
    # the device-side start of the basis: Q = I, then rounds of (sort, power iteration, QR) - orthogonal
    # iteration.  The oracle takes the same steps; after a few rounds the leading columns are the leading
    # eigenvectors of the oracle's Jacobi decomposition.
    n, rounds = 160, 6
    lam = torch.cat([torch.tensor([10.0, 5.0, 2.5, 1.2], device=DEV, dtype=torch.float64),
                     torch.linspace(0.1, 0.01, n - 4, device=DEV, dtype=torch.float64)])
    A, _ = spectrum_factor(n, lam, 420)
    Q = torch.full((n, n), float("nan"), device=DEV)                  # ignored: the call starts from the identity
    info = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    ast.soap_refresh([(A, Q)], info=info, sort=True, from_identity=True, rounds=rounds)
    torch.cuda.synchronize()
    assert info.item() == 0
    Qo = np.eye(n)
    for _ in range(rounds):
        Qo, _, _ = oracle.soap_sort(np64(A), Qo)
        Qo, _ = oracle.soap_refresh(np64(A), Qo)
    q = np64(Q)
    assert np.linalg.norm(q.T @ q - np.eye(n)) / math.sqrt(n) <= 1e-5
    assert np.all(np.abs(np.sum(q[:, :4] * Qo[:, :4], axis=0)) >= 0.999)
    lamJ, VJ, _ = oracle.jacobi_eigh(np64(A))
    order = np.argsort(-lamJ)
    assert np.all(np.abs(np.sum(q[:, :4] * VJ[:, order[:4]], axis=0)) >= 0.999)


def test_soap_reproject_carries_the_moments_to_the_new_bases():
    shapes = [(200, 328), (64, 64), (257, 130), (1, 5)]
    items, refs, keep = [], [], []
    for i, (m, n) in enumerate(shapes):
        QLo, QLn = W.haar(m, DEV, 500 + i), W.haar(m, DEV, 510 + i)
        QRo, QRn = W.haar(n, DEV, 520 + i), W.haar(n, DEV, 530 + i)
        M = padded(m, n, 3); M.copy_(W.gaussian_block(m, n, 1.0, DEV, 540 + i))
        V = padded(m, n, 1); V.copy_(W.gaussian_block(m, n, 1.0, DEV, 550 + i) ** 2)
        g = torch.Generator(device=DEV).manual_seed(60 + i)
        pl = torch.randperm(m, device=DEV, generator=g).to(torch.int32)
        pr = torch.randperm(n, device=DEV, generator=g).to(torch.int32)
        refs.append((oracle.soap_reproject(np64(M), np64(QLo), np64(QRo), np64(QLn), np64(QRn)),
                     np64(V)[pl.cpu().numpy().astype(np.int64)][:, pr.cpu().numpy().astype(np.int64)]))
        items.append((QLo, QLn, QRo, QRn, M, V, pl, pr if i != 1 else None))
        if i == 1:
            refs[-1] = (refs[-1][0], np64(V)[pl.cpu().numpy().astype(np.int64)])
    ast.soap_reproject(items)
    torch.cuda.synchronize()
    for (QLo, QLn, QRo, QRn, M, V, pl, pr), (Mo, Vo) in zip(items, refs):
        print("reproject", tuple(M.shape), relF(M, Mo))
        assert relF(M, Mo) <= 1e-4                    # two bf16 terms per operand: 16 bits kept
        assert np.array_equal(np64(V), Vo)            # a pure reordering
        assert torch.all(M._base[:, M.shape[1]:] == -777.0) and torch.all(V._base[:, V.shape[1]:] == -777.0)
    # only V, only M
    m, n = 40, 24
    V = W.gaussian_block(m, n, 1.0, DEV, 570); V0 = V.clone()
    pl = torch.arange(m - 1, -1, -1, device=DEV, dtype=torch.int32)
    ast.soap_reproject([(None, None, None, None, None, V, pl, None)])
    torch.cuda.synchronize()
    assert torch.equal(V, V0.flip(0))


def test_soap_refresh_rank_deficient_products():
    # A Q of rank < n: a numerically dependent column (m x m statistic of one m x n gradient, n < m)
    # still yields an orthogonal Q whose leading columns are the oracle's - what is left of such a
    # column after the projections is round-off, normalised to some unit vector and orthogonalised
    # again by the second sweep; a column that is exactly zero cannot be normalised and fails its
    # factor, and only that factor
    n = 64
    A1 = torch.zeros(n, n, device=DEV); A1[:40, :40] = spd(40, 7)
    G = W.gaussian_block(200, 136, 1.0, DEV, 8)
    A2 = (0.05 * G @ G.T).contiguous()
    A3 = spd(96, 9)
    G4 = W.gaussian_block(512, 64, 1.0, DEV, 10)          # rank 64 of 512: three of four panels are round-off
    A4 = (0.05 * G4 @ G4.T).contiguous()
    Qs = [torch.eye(n, device=DEV), torch.eye(200, device=DEV), torch.eye(96, device=DEV), torch.eye(512, device=DEV)]
    info = torch.full((4,), -1, dtype=torch.int32, device=DEV)
    ast.soap_refresh([(A1, Qs[0]), (A2, Qs[1]), (A3, Qs[2]), (A4, Qs[3])], info=info)
    torch.cuda.synchronize()
    info = info.cpu().numpy()
    assert info[0] == B.INFO_NOT_PD and np.all(info[1:] == B.INFO_OK), info
    for A, Q in ((A2, Qs[1]), (A3, Qs[2]), (A4, Qs[3])):
        k = Q.shape[0]
        q = np64(Q)
        assert np.linalg.norm(q.T @ q - np.eye(k)) / math.sqrt(k) <= 1e-5
        Qo, _ = oracle.soap_refresh(np64(A), np.eye(k))
        assert np.all(np.sum(q[:, :32] * Qo[:, :32], axis=0) >= 0.999)


# =============================================================================== a5 SOAP step

def test_soap_step_same_basis_parity_over_three_steps():
    shapes = [(128, 128, torch.float32), (200, 328, torch.bfloat16), (257, 64, torch.bfloat16)]
    state = []
    for i, (m, n, dt) in enumerate(shapes):
        QL, QR = W.haar(m, DEV, 80 + i), W.haar(n, DEV, 90 + i)
        M = torch.zeros(m, n, device=DEV); V = torch.zeros(m, n, device=DEV); N = padded(m, n, 1)
        state.append((QL, QR, M, V, N, np.zeros((m, n)), np.zeros((m, n))))
    for t in (1, 2, 3):
        items, Gs = [], []
        for i, (m, n, dt) in enumerate(shapes):
            QL, QR, M, V, N, _, _ = state[i]
            U, Vb = W.haar(m, DEV, 100 + i), W.haar(n, DEV, 110 + i)
            G = W.soap_gradient(U, Vb, t, DEV, i, dtype=dt)
            Gs.append(G)
            items.append((G, QL, QR, M, V, N))
        Min = [np64(s[2]) for s in state]; Vin = [np64(s[3]) for s in state]
        ast.soap_step(items, 0.9, 0.95, 1e-8, t)
        torch.cuda.synchronize()
        for i in range(len(shapes)):
            QL, QR, M, V, N, _, _ = state[i]
            No, Mo, Vo = oracle.soap_step(np64(Gs[i]), np64(QL), np64(QR), Min[i], Vin[i], 0.9, 0.95, 1e-8, t)
            # the rotations keep 16 bits of Q_L, Q_R and of the intermediate product (two bf16 terms
            # each): the rotated gradient, and with it the moments, carry a few 2^-16 of relative error
            assert relF(M, Mo) <= 2e-4 and relF(V, Vo) <= 2e-4
            assert relF(N, No) <= TOL_PRECOND, (t, i, relF(N, No))
            assert torch.all(N._base[:, N.shape[1]:] == -777.0)


def test_soap_step_whole_tile_blocks_mixed_with_ragged_ones():
    # whole 256 x 256 tiles: the three split x split products of each rotation pair run on the
    # 8-wavefront kernel (one of them storing transposed); the ragged block keeps the other path
    shapes = [(256, 512, torch.float32), (200, 328, torch.bfloat16), (512, 256, torch.bfloat16), (256, 256, torch.bfloat16)]
    state = []
    for i, (m, n, dt) in enumerate(shapes):
        QL, QR = W.haar(m, DEV, 180 + i), W.haar(n, DEV, 190 + i)
        M = torch.zeros(m, n, device=DEV); V = torch.zeros(m, n, device=DEV); N = padded(m, n, 4 if i != 3 else 1)
        state.append((QL, QR, M, V, N))
    for t in (1, 2):
        items, Gs = [], []
        for i, (m, n, dt) in enumerate(shapes):
            QL, QR, M, V, N = state[i]
            U, Vb = W.haar(m, DEV, 200 + i), W.haar(n, DEV, 210 + i)
            G = W.soap_gradient(U, Vb, t, DEV, i, dtype=dt)
            Gs.append(G)
            items.append((G, QL, QR, M, V, N))
        Min = [np64(s[2]) for s in state]; Vin = [np64(s[3]) for s in state]
        ast.soap_step(items, 0.9, 0.95, 1e-8, t)
        torch.cuda.synchronize()
        for i in range(len(shapes)):
            QL, QR, M, V, N = state[i]
            No, Mo, Vo = oracle.soap_step(np64(Gs[i]), np64(QL), np64(QR), Min[i], Vin[i], 0.9, 0.95, 1e-8, t)
            print("soap step whole tiles", shapes[i], t, relF(M, Mo), relF(V, Vo), relF(N, No))
            assert relF(M, Mo) <= 2e-4 and relF(V, Vo) <= 2e-4
            assert relF(N, No) <= TOL_PRECOND, (t, i, relF(N, No))
            assert torch.all(N._base[:, N.shape[1]:] == -777.0)


def test_soap_step_one_sided_blocks():
    # a block that keeps a basis on one side only (the other dimension is above the preconditioner cap):
    # QL or QR absent stands for the identity; mixed with a two-sided block in one call
    cases = [(200, 328, torch.bfloat16, "L"), (129, 70, torch.float32, "R"), (64, 256, torch.float32, "L"),
             (257, 130, torch.bfloat16, "R"), (128, 128, torch.bfloat16, "LR")]
    state = []
    for i, (m, n, dt, side) in enumerate(cases):
        QL = W.haar(m, DEV, 600 + i) if "L" in side else None
        QR = W.haar(n, DEV, 610 + i) if "R" in side else None
        M = torch.zeros(m, n, device=DEV); V = torch.zeros(m, n, device=DEV); N = padded(m, n, 2)
        state.append((QL, QR, M, V, N))
    for t in (1, 2):
        items, Gs = [], []
        for i, (m, n, dt, side) in enumerate(cases):
            QL, QR, M, V, N = state[i]
            G = W.soap_gradient(W.haar(m, DEV, 620 + i), W.haar(n, DEV, 630 + i), t, DEV, i, dtype=dt)
            Gs.append(G)
            items.append((G, QL, QR, M, V, N))
        Min = [np64(s[2]) for s in state]; Vin = [np64(s[3]) for s in state]
        ast.soap_step(items, 0.9, 0.95, 1e-8, t)
        torch.cuda.synchronize()
        for i, (m, n, dt, side) in enumerate(cases):
            QL, QR, M, V, N = state[i]
            ql = np64(QL) if QL is not None else np.eye(m)
            qr = np64(QR) if QR is not None else np.eye(n)
            No, Mo, Vo = oracle.soap_step(np64(Gs[i]), ql, qr, Min[i], Vin[i], 0.9, 0.95, 1e-8, t)
            print("one-sided soap step", cases[i], t, relF(M, Mo), relF(V, Vo), relF(N, No))
            assert relF(M, Mo) <= 2e-4 and relF(V, Vo) <= 2e-4 and relF(N, No) <= TOL_PRECOND
            assert torch.all(N._base[:, N.shape[1]:] == -777.0)


def test_soap_step_with_transposed_bases_kept_by_the_caller_is_bit_identical():
    """Q_L^T and Q_R^T passed in the block (asteria_transpose, once per refresh) instead of transposed by
    every step: same products on the same values, so the results must agree bit for bit; and the utility
    against the definition, on ragged shapes with padded leading dimensions."""
    src = padded(70, 133, 5); src.copy_(W.gaussian_block(70, 133, 1.0, DEV, 91))
    dst = padded(133, 70, 3)
    ast.transpose([(src, dst)])
    torch.cuda.synchronize()
    assert torch.equal(dst, src.T)
    shapes = [(200, 328), (256, 512), (129, 70)]
    Gs = [W.gaussian_block(m, n, 1.0, DEV, 92, i, dtype=torch.bfloat16) for i, (m, n) in enumerate(shapes)]
    QLs = [W.haar(m, DEV, 93, i) for i, (m, n) in enumerate(shapes)]
    QRs = [W.haar(n, DEV, 94, i) for i, (m, n) in enumerate(shapes)]
    QLt = [torch.empty_like(q) for q in QLs]; QRt = [torch.empty_like(q) for q in QRs]
    ast.transpose(list(zip(QLs, QLt)) + list(zip(QRs, QRt)))
    out = []
    for cached in (False, True):
        Ms = [torch.zeros(m, n, device=DEV) for m, n in shapes]
        Vs = [torch.zeros(m, n, device=DEV) for m, n in shapes]
        Ns = [torch.full((m, n), float("nan"), device=DEV) for m, n in shapes]
        items = list(zip(Gs, QLs, QRs, Ms, Vs, Ns, QLt, QRt)) if cached else list(zip(Gs, QLs, QRs, Ms, Vs, Ns))
        need = [ast.soap_step_workspace_bytes(items)]
        for t in (1, 2):
            ast.soap_step(items, 0.9, 0.95, 1e-8, t)
        torch.cuda.synchronize()
        out.append((Ms, Vs, Ns, need[0]))
    for a, b in zip(out[0][:3], out[1][:3]):
        assert all(torch.equal(x, y) for x, y in zip(a, b))
    assert out[1][3] < out[0][3]                       # and the workspace no longer holds the copies
    # only one of the two kept: the other is still made by the call
    Ms = [torch.zeros(m, n, device=DEV) for m, n in shapes]
    Vs = [torch.zeros(m, n, device=DEV) for m, n in shapes]
    Ns = [torch.full((m, n), float("nan"), device=DEV) for m, n in shapes]
    items = list(zip(Gs, QLs, QRs, Ms, Vs, Ns, QLt, [None] * 3))
    for t in (1, 2):
        ast.soap_step(items, 0.9, 0.95, 1e-8, t)
    torch.cuda.synchronize()
    assert all(torch.equal(x, y) for x, y in zip(Ns, out[0][2]))


def test_soap_step_identity_bases_reduce_to_adam():
    m, n = 33, 65
    G = W.gaussian_block(m, n, 0.02, DEV, 120)
    M = torch.zeros(m, n, device=DEV); V = torch.zeros(m, n, device=DEV); N = torch.empty(m, n, device=DEV)
    ast.soap_step([(G, torch.eye(m, device=DEV), torch.eye(n, device=DEV), M, V, N)], 0.9, 0.95, 1e-8, 1)
    torch.cuda.synchronize()
    g = np64(G)
    assert relF(N, g / (np.abs(g) + 1e-8)) <= 1e-4      # 16 bits of every operand are kept (two bf16 terms)


# =============================================================================== degenerate shapes

def test_tiny_and_vector_shaped_blocks_through_every_entry_point():
    """1 x 1, 1 x n, m x 1 and 2 x 3 blocks (a 1-D slice of a blocked matrix is such a block): every
    stage against the oracle, all shapes in one batch beside an ordinary block."""
    shapes = [(1, 1), (1, 37), (45, 1), (2, 3), (130, 70)]
    Gs = [W.gaussian_block(m, n, 1.0, DEV, 77, i) for i, (m, n) in enumerate(shapes)]
    Ls = [torch.eye(m, device=DEV) for m, n in shapes]
    Rs = [torch.eye(n, device=DEV) for m, n in shapes]
    L0 = [np64(x) for x in Ls]; R0 = [np64(x) for x in Rs]
    ast.stats_update(list(zip(Gs, Ls, Rs)), 0.95)
    torch.cuda.synchronize()
    for G, L, R, l0, r0 in zip(Gs, Ls, Rs, L0, R0):
        Lo, Ro = oracle.stats_update(np64(G), l0, r0, 0.95)
        assert relF(L, Lo) <= TOL_STATS and relF(R, Ro) <= TOL_STATS
    As = Ls + Rs
    Xs, info, iters, _, lmax = run_roots(As, 1e-6)
    assert np.all(info == B.INFO_OK), info
    for A, X, lm in zip(As, Xs, lmax):
        Xo, lmo, _ = oracle.inverse_root(np64(A), 1e-6)
        assert relF(X, Xo) <= TOL_ROOT, (tuple(A.shape), relF(X, Xo))
        assert abs(lm - lmo) <= 1e-3 * lmo
    k = len(shapes)
    Ps = [torch.full((m, n), float("nan"), device=DEV) for m, n in shapes]
    ast.precondition(list(zip(Xs[:k], Gs, Xs[k:], Ps)))
    torch.cuda.synchronize()
    for XL, G, XR, P in zip(Xs[:k], Gs, Xs[k:], Ps):
        assert relF(P, oracle.precondition(np64(XL), np64(G), np64(XR))) <= TOL_PRECOND
    # SOAP: refresh from the identity, then one step with the refreshed bases
    Qs = [torch.eye(A.shape[0], device=DEV) for A in As]
    qinfo = torch.full((2 * k,), -1, dtype=torch.int32, device=DEV)
    ast.soap_refresh(list(zip(As, Qs)), info=qinfo)
    torch.cuda.synchronize()
    assert np.all(qinfo.cpu().numpy() == B.INFO_OK)
    for A, Q in zip(As, Qs):
        n = A.shape[0]
        Qo, _ = oracle.soap_refresh(np64(A), np.eye(n))
        q = np64(Q)
        assert np.linalg.norm(q.T @ q - np.eye(n)) / n ** 0.5 <= 1e-5
        assert np.linalg.norm(q[:, :1] - Qo[:, :1]) <= 1e-4          # leading column (the whole basis for n = 1)
    Ms = [torch.zeros(m, n, device=DEV) for m, n in shapes]
    Vs = [torch.zeros(m, n, device=DEV) for m, n in shapes]
    Ns = [torch.full((m, n), float("nan"), device=DEV) for m, n in shapes]
    ast.soap_step(list(zip(Gs, Qs[:k], Qs[k:], Ms, Vs, Ns)), 0.9, 0.95, 1e-8, 1)
    torch.cuda.synchronize()
    for i, (m, n) in enumerate(shapes):
        No, Mo, Vo = oracle.soap_step(np64(Gs[i]), np64(Qs[i]), np64(Qs[k + i]), np.zeros((m, n)), np.zeros((m, n)),
                                      0.9, 0.95, 1e-8, 1)
        assert relF(Ms[i], Mo) <= 2e-4 and relF(Vs[i], Vo) <= 2e-4, shapes[i]
        assert relF(Ns[i], No) <= TOL_PRECOND, (shapes[i], relF(Ns[i], No))


# =============================================================================== determinism

def test_two_runs_are_bit_identical():
    n = 200
    G = W.lowrank_block(n, n, DEV, 130)
    outs = []
    for _ in range(2):
        L = torch.zeros(n, n, device=DEV); R = torch.zeros(n, n, device=DEV)
        ast.stats_update([(G, L, R)], 0.95)
        (XL, XR), info, iters, _, _ = run_roots([L, R], 1e-6)
        P = torch.empty(n, n, device=DEV)
        ast.precondition([(XL, G, XR, P)])
        torch.cuda.synchronize()
        outs.append((L.clone(), XL.clone(), XR.clone(), P.clone(), iters.copy()))
    for a, b in zip(outs[0][:4], outs[1][:4]):
        assert torch.equal(a, b)
    assert np.array_equal(outs[0][4], outs[1][4])
