"""Writes the stored expected values of the ill-conditioned stress workload (8 blocks of
4096 x 4096, singular values log-spaced over 8 decades, bf16 gradients, fp32 statistics,
eps = 1e-8 lambda_max) for ONE block: both of its factors, n = 4096.

The cyclic-Jacobi oracle needs a few hours per factor at this size, too long for a test run, so
its answer is computed once here and a sample of it is stored:

  cfg5_block<b>.npz   per side s in {L, R}:
      rows_s    int64[32]        seeded row indices
      A_rows_s  float32[32, n]   those rows of the fp32 statistic the root is taken of
      X_rows_s  float64[32, n]   the same rows of X = (A + eps I)^(-1/4), eps = 1e-8 lambda_max
      lam_s     float64[n]       Jacobi's spectrum of A (unsorted)
      P_rows    float64[32, n]   rows rows_L of P = X_L G X_R (paper Eq. 1) from the two oracle roots
  cfg5_block<b>.json  seeds, sizes, lambda_max, oracle status, sha256 of the gradient's bf16 bits
                      and of the fp32 statistics, timings

Everything stored is computed by `oracle/` (float64 statistics by triple loops, rounded to fp32
as the workload says "fp32 statistics"; Jacobi; spectral root) from the numpy PCG64 inputs of
`workloads_np.py`, which is loaded by file path so that the HIP library is never loaded in this
process.  Nothing here touches a GPU.  What the operations are: paper Sec. I / Sec. III-B (the
statistics L, R), Eq. 1 (their inverse 4th roots).

Run (from the repository root):  python tests/golden/make_cfg5_fixture.py [--n 4096] [--block 0]
"""
from __future__ import annotations

import argparse
import hashlib
import importlib.util
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402

_spec = importlib.util.spec_from_file_location(
    "workloads_np", os.path.join(ROOT, "paper_2605_16184_amd", "workloads_np.py"))
WN = importlib.util.module_from_spec(_spec)
_spec.loader.exec_module(WN)

CFG = 5
# beta and eps as the fp32 numbers the C ABI carries (1 - beta is then exact in fp32 too), so that the
# stored statistics are the ones a float64 accumulation of the same call arguments rounds to
BETA = float(np.float32(0.95))
EPS_REL = float(np.float32(1e-8))
NROWS = 32


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=4096)
    ap.add_argument("--block", type=int, default=0)
    ap.add_argument("--out", default=HERE)
    args = ap.parse_args()
    n, b = args.n, args.block

    t0 = time.time()
    G = WN.logspaced_block(CFG, b, n=n, decades=8.0)
    g_sha = hashlib.sha256(WN.bf16_bits(G).tobytes()).hexdigest()
    print(f"[fixture] G {n}x{n} generated in {time.time() - t0:.1f} s, sha256 {g_sha[:16]}", flush=True)

    t0 = time.time()
    L64, R64 = oracle.stats_update(G, np.zeros((n, n)), np.zeros((n, n)), BETA)
    t_stats = time.time() - t0
    A = {"L": L64.astype(np.float32), "R": R64.astype(np.float32)}   # "fp32 statistics"
    print(f"[fixture] oracle statistics in {t_stats:.1f} s", flush=True)

    def root(side: str):
        t = time.time()
        st, X, lmax, lam = oracle.inverse_root(A[side].astype(np.float64), EPS_REL, relative=True,
                                               return_status=True)
        dt = time.time() - t
        print(f"[fixture] side {side}: oracle status {st}, lambda_max {lmax:.9e}, "
              f"lambda_min/lambda_max {lam.min() / lmax:.3e}, {dt:.0f} s", flush=True)
        return st, X, lmax, lam, dt

    with ThreadPoolExecutor(max_workers=2) as ex:
        res = dict(zip("LR", ex.map(root, "LR")))

    arrays, meta = {}, {
        "what": "inverse 4th roots (paper Eq. 1) of the fp32 statistics (paper Sec. I, III-B) of one "
                "block of the ill-conditioned stress workload, by the float64 cyclic-Jacobi oracle",
        "written_by": "tests/golden/make_cfg5_fixture.py",
        "seed": [WN.SEED0, CFG, b, 0], "n": n, "beta": BETA, "eps_rel": EPS_REL,
        "G_bf16_sha256": g_sha, "oracle_stats_seconds": round(t_stats, 1), "sides": {}}
    for s, (side, (st, X, lmax, lam, dt)) in enumerate(res.items()):
        rows = WN.sample_rows(CFG, b, s, n, min(NROWS, n))
        arrays[f"rows_{side}"] = rows.astype(np.int64)
        arrays[f"A_rows_{side}"] = A[side][rows]
        arrays[f"X_rows_{side}"] = X[rows]
        arrays[f"lam_{side}"] = lam
        meta["sides"][side] = {
            "oracle_status": int(st), "lambda_max": float(lmax), "lambda_min": float(lam.min()),
            "A_f32_sha256": hashlib.sha256(A[side].tobytes()).hexdigest(),
            "X_fro": float(np.linalg.norm(X)) if st == oracle.OK else None,
            "oracle_seconds": round(dt, 1)}
    if all(r[0] == oracle.OK for r in res.values()):
        t0 = time.time()
        P = oracle.precondition(res["L"][1], G, res["R"][1])
        arrays["P_rows"] = P[arrays["rows_L"]]
        meta["P_fro"] = float(np.linalg.norm(P))
        print(f"[fixture] oracle precondition in {time.time() - t0:.0f} s", flush=True)
    tag = f"cfg5_block{b}" + ("" if n == 4096 else f"_n{n}")
    np.savez(os.path.join(args.out, tag + ".npz"), **arrays)
    with open(os.path.join(args.out, tag + ".json"), "w") as f:
        json.dump(meta, f, indent=1)
    print(f"[fixture] wrote {tag}.npz / .json", flush=True)


if __name__ == "__main__":
    main()
