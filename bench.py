#!/usr/bin/env python3
"""Benchmark of the Shampoo preconditioner hot path on one MI355X.

Workload (the configuration the headline metric is quoted on): every 2-D gradient of a 1.1B
LLaMA-style model (d=2048, 22 layers, FFN 5632, vocab 32000; 1 099 956 224 parameters) blocked
at <= 1024 x 1024 -> 1184 blocks, 2368 Kronecker factors; synthetic bf16 gradients with
power-law singular values (sigma_i ~ 1/i), beta = 0.95, eps = 1e-6 lambda_max.

One "step" = one pass of the whole path over that batch, inputs resident in HBM:
    asteria_stats_update (all blocks) -> asteria_inverse_root (all factors, the "full
    preconditioner refresh") -> asteria_precondition (all blocks).
`value` = milliseconds per full refresh (the inverse-root call over all factors);
`ms_per_step` = the whole pass.  Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_F32_MFMA = 157.3   # TFLOP/s, MI355X dense fp32 matrix
PEAK_F64_MFMA = 78.6    # TFLOP/s, MI355X dense fp64 matrix
PEAK_BF16_MFMA = 2500.0 # TFLOP/s, MI355X dense bf16 and fp16 matrix
PEAK_I8_MFMA = 5000.0   # TOP/s, MI355X dense int8 matrix
# What a register-only loop of v_mfma_f64_16x16x4_f64 with random operands sustains on the box
# (2 or 4 wavefronts per SIMD, 8 independent accumulators each, 2.38 GHz): context for the fp64
# kernel's fraction of the published peak, never used as `peak`.
MEASURED_F64_MFMA_LOOP = 58.8
PEAK_HBM = 8000.0       # GB/s


def stored_traffic(key: str):
    """HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (each scaled by a
    plain copy of known size); the runs and their summary live under profiles/."""
    import re
    path = os.path.join(ROOT, "profiles", "gemm_grouped__llama1b_b1024_hbm_traffic.md")
    try:
        m = re.search(rf"{key}\s*=\s*([0-9.eE+-]+)", open(path).read())
        return float(m.group(1)) if m else None
    except OSError:
        return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def sym_gemm_flops(n: int) -> float:
    """Algorithmic flops of one symmetric n x n x n product when only one triangle is computed."""
    return float(n) * (n + 1) * n


def newton_gemm_counts(iters: int, j64: int, jlow: int, xt_lowp: bool):
    """(fp32 GEMMs, fp64 GEMMs, split-fp16 GEMMs) a factor executed: iteration k < iters does
    X <- X T (except k = 0, where X_1 is written by the start kernel), and for k < iters - 1 also
    the M-chain T^2, T^4 and T^4 M; the chain runs on the fp64 cores for k < j64 and on the fp16
    cores (two-term split operands) for k >= jlow; X <- X T runs there too when xt_lowp, else with its iteration's
    tier (fp32 at least)."""
    g32 = g64 = g16 = 0
    for k in range(iters):
        chain = 3 if k < iters - 1 else 0
        lowp = k >= max(jlow, j64)
        if k < j64:
            g64 += chain
        elif lowp:
            g16 += chain
        else:
            g32 += chain
        if k > 0:
            if xt_lowp or lowp:
                g16 += 1
            else:
                g32 += 1
    return g32, g64, g16


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--ws-gib", type=float, default=128.0, help="workspace handed to the library (a single pass needs about 107 GiB)")
    ap.add_argument("--max-blocks", type=int, default=0, help="debug: truncate the batch")
    ap.add_argument("--fp64-iters", type=int, default=-1)
    ap.add_argument("--lowp-from", type=int, default=-1, help="first iteration on the fp16 cores with split operands (-1 = library rule)")
    ap.add_argument("--int8-slices", type=int, default=-1, help="products of the fp64 iterations: -1 = library default (int8 cores, 5 slices), 0 = fp64 cores, 4 | 5")
    ap.add_argument("--schedule", type=int, default=1, help="1 = interval-adapted coefficients, 0 = classical Newton")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-soap", action="store_true", help="skip the SOAP section (blocks <= 2048)")
    ap.add_argument("--gaussian-inputs", action="store_true",
                    help="plain N(0, 0.01^2) gradients instead of power-law spectra (counter runs: no QR in the generator)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no collectives or sharding in this library).", file=sys.stderr)
        return 2

    import torch
    import paper_2605_16184_amd as ast
    from paper_2605_16184_amd import workloads as W

    dev = "cuda:0"
    torch.cuda.set_device(0)
    beta, eps_rel = 0.95, 1e-6

    shapes = W.block_shapes(W.llama_1b_matrices(), 1024)
    if args.max_blocks:
        shapes = shapes[:: max(1, len(shapes) // args.max_blocks)][: args.max_blocks]
    by_shape, by_factor, params = W.census(shapes)
    log(f"[bench] {len(shapes)} blocks, factors {by_factor}, {params} parameters")

    t0 = time.time()
    if args.gaussian_inputs:
        Gs = [W.gaussian_block(m, n, 0.01, dev, 3, b, dtype=torch.bfloat16) for b, (m, n) in enumerate(shapes)]
    else:
        Gs = W.powerlaw_blocks(shapes, dev)
    Ls = [torch.zeros(m, m, device=dev) for m, n in shapes]
    Rs = [torch.zeros(n, n, device=dev) for m, n in shapes]
    XLs = [torch.empty(m, m, device=dev) for m, n in shapes]
    XRs = [torch.empty(n, n, device=dev) for m, n in shapes]
    Ps = [torch.empty(m, n, device=dev) for m, n in shapes]
    torch.cuda.synchronize()
    log(f"[bench] inputs generated on the GPU in {time.time() - t0:.1f} s; "
        f"{torch.cuda.memory_allocated() / 2**30:.1f} GiB resident")

    blocks = ast.Blocks(list(zip(Gs, Ls, Rs)))
    factors = ast.Factors([(L, X) for L, X in zip(Ls, XLs)] + [(R, X) for R, X in zip(Rs, XRs)])
    pblocks = ast.PBlocks(list(zip(XLs, Gs, XRs, Ps)))
    nf = len(factors)
    fsize = [m for m, n in shapes] + [n for m, n in shapes]
    opts = ast.RootOpts(fp64_iters=args.fp64_iters, schedule=args.schedule, lowp_from=args.lowp_from,
                        int8_slices=args.int8_slices)
    full, mn = ast.inverse_root_workspace_bytes(factors, opts)
    ws_bytes = int(max(min(full, args.ws_gib * 2**30), mn, ast.precondition_workspace_bytes(pblocks),
                       ast.stats_update_workspace_bytes(blocks)))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    info = torch.zeros(nf, dtype=torch.int32, device=dev)
    iters = torch.zeros(nf, dtype=torch.int32, device=dev)
    resid = torch.zeros(nf, device=dev)
    log(f"[bench] workspace {ws_bytes / 2**30:.1f} GiB (single pass would need {full / 2**30:.1f} GiB)")

    def one_step(ev=None):
        if ev: ev[0].record()
        ast.stats_update(blocks, beta, ws=ws)
        if ev: ev[1].record()
        ast.inverse_root(factors, eps_rel, relative=True, root=4, opts=opts, info=info, iters=iters,
                         resid=resid, ws=ws)
        if ev: ev[2].record()
        ast.precondition(pblocks, ws=ws)
        if ev: ev[3].record()

    if args.calibrate_copy:
        src = torch.empty(2**28, dtype=torch.float32, device=dev).fill_(1.0)    # 1 GiB
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for w in range(args.warmup):
        t = time.time()
        one_step()
        torch.cuda.synchronize()
        log(f"[bench] warmup {w}: {1e3 * (time.time() - t):.0f} ms")

    # precision schedule the library uses for these options (for flop accounting)
    j64, jlow, xt_lowp = ast.inverse_root_plan(eps_rel, relative=True, root=4, opts=opts)

    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    ast.profile_enable(200000)
    flops32 = flops64 = flops16 = 0.0
    torch.cuda.synchronize()
    t_wall = time.time()
    for s in range(args.steps):
        one_step(evs[s])
        torch.cuda.synchronize()          # step boundary (also lets the iteration counts be read)
        it = iters.cpu().numpy()
        for n, c in zip(fsize, it):
            g32, g64, g16 = newton_gemm_counts(int(c), j64, jlow, xt_lowp)
            flops32 += g32 * sym_gemm_flops(n)
            flops64 += g64 * sym_gemm_flops(n)
            flops16 += g16 * sym_gemm_flops(n)
        log(f"[bench] step {s}: {evs[s][0].elapsed_time(evs[s][3]):.0f} ms")
    wall_ms = 1e3 * (time.time() - t_wall)
    prof = ast.profile_collect(200000)

    stats_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps
    refresh_ms = sum(e[1].elapsed_time(e[2]) for e in evs) / args.steps
    precond_ms = sum(e[2].elapsed_time(e[3]) for e in evs) / args.steps
    step_ms = sum(e[0].elapsed_time(e[3]) for e in evs) / args.steps
    info_h = info.cpu().numpy()
    it = iters.cpu().numpy()

    k32 = [ms for ms, kind in prof if kind == 0]
    k64 = [ms for ms, kind in prof if kind == 1]
    k16 = [ms for ms, kind in prof if kind == 224]       # 16-bit cores, both operands fp32 split in two fp16 terms
    k8 = [ms for ms, kind in prof if kind in (304, 305)]  # int8 cores: fp64 operands as diagonal + 7-bit slices
    t8 = sum(k8) * 1e-3
    # int8 MFMA passes per product: 10 with 4 slices, 15 with 5; the count is chosen per factor and
    # product on the device and not reported to the host, so the issue rate below is a lower bound
    passes8 = 10.0
    # the fp64 launches that follow the int8 ones take the products the device-side estimate declined;
    # when they are (nearly) empty the flops of the fp64 iterations were done on the int8 cores
    on_i8 = t8 > 0 and sum(k64) * 1e-3 < 0.05 * t8
    flops8 = flops64 if on_i8 else 0.0
    if on_i8: flops64 = 0.0
    tf8 = flops8 / t8 / 1e12 if t8 > 0 else 0.0
    t16 = sum(k16) * 1e-3
    tf16 = flops16 / t16 / 1e12 if t16 > 0 else 0.0
    t32, t64 = sum(k32) * 1e-3, sum(k64) * 1e-3
    tf32 = flops32 / t32 / 1e12 if t32 > 0 else 0.0
    tf64 = flops64 / t64 / 1e12 if t64 > 0 else 0.0
    stats_flops = sum(sym_gemm_flops(m) / m * n + sym_gemm_flops(n) / n * m for m, n in shapes)
    stats_bytes = sum(2 * m * n + 8 * (m * m + n * n) for m, n in shapes)
    precond_flops = sum(2.0 * m * n * (m + n) for m, n in shapes)
    precond_issued = sum(2.0 * (2.0 * m * n * n) + 3.0 * (2.0 * m * m * n) for m, n in shapes)
    precond_bytes = sum(4 * m * m + 4 * n * n + 2 * m * n + 4 * m * n for m, n in shapes)
    log(f"[bench] stats {stats_ms:.2f} ms  refresh {refresh_ms:.1f} ms  precondition {precond_ms:.2f} ms")
    log(f"[bench] fp32 GEMM: {len(k32)} launches, {t32 * 1e3:.1f} ms total, {tf32:.1f} TFLOP/s algorithmic; "
        f"fp64 GEMM: {len(k64)} launches, {t64 * 1e3:.1f} ms total, {tf64:.1f} TFLOP/s; "
        f"split-fp16 GEMM: {len(k16)} launches, {t16 * 1e3:.1f} ms total, {tf16:.1f} fp32-equivalent TFLOP/s; "
        f"int8-slice GEMM: {len(k8)} launches, {t8 * 1e3:.1f} ms total, {tf8:.1f} fp64-equivalent TFLOP/s")
    log(f"[bench] Newton iterations min/mean/max {it.min()}/{it.mean():.1f}/{it.max()}, info!=0: {(info_h != 0).sum()}")

    out = {
        "metric": "ms per full preconditioner refresh (1B model) + % MFMA peak; ms per step",
        "value": round(refresh_ms, 3),
        "unit": "ms per full refresh (inverse 4th roots of all 2368 factors)",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(step_ms, 3),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "1.1B LLaMA-style model, all 2-D grads blocked at <=1024 (1184 blocks, 2368 factors), "
                               "bf16 power-law gradients, fp32 statistics, eps=1e-6*lambda_max, beta=0.95",
                   "blocks": len(shapes), "factors": nf, "fp64_prefix_iters": j64, "fp64_prefix_products": ("fp64 cores" if args.int8_slices == 0 else
                                                                      "int8 cores, diagonal + 7-bit slices (fp64 cores where the device-side estimate declines)"),
                   "fp16_split_from_iter": jlow, "x_update_on_fp16_cores": xt_lowp,
                   "schedule": "interval-adapted" if args.schedule == 1 else "classical Newton",
                   "workspace_gib": round(ws_bytes / 2**30, 1)},
        "breakdown_ms": {"stats_update": round(stats_ms, 3), "inverse_root": round(refresh_ms, 3),
                         "precondition": round(precond_ms, 3), "step_excl_refresh": round(stats_ms + precond_ms, 3),
                         "amortised_step_pf10": round(stats_ms + precond_ms + refresh_ms / 10, 3)},
        "newton_iters": {"min": int(it.min()), "mean": round(float(it.mean()), 2), "max": int(it.max())},
        "not_converged": int((info_h != 0).sum()),
        "wall_ms_timed_region": round(wall_ms, 1),
        "roofline_fp32": {"kernel": "gemm_grouped_kernel<float> (symmetric fp32-MFMA products of the root iteration)",
                          "bound": "mfma", "achieved": round(tf32, 2), "peak": PEAK_F32_MFMA, "unit": "TFLOP/s",
                          "frac": round(tf32 / PEAK_F32_MFMA, 4), "traffic": stored_traffic("traffic_bytes_per_launch_fp32"),
                          "launches": len(k32), "avg_launch_ms": round(1e3 * t32 / max(len(k32), 1), 4),
                          "flops_per_launch": round(flops32 / max(len(k32), 1), 1)},
        "roofline_fp64": {"kernel": "gemm_grouped_kernel<double> (fp64-MFMA products of the leading root iterations)",
                          "bound": "mfma", "achieved": round(tf64, 2), "peak": PEAK_F64_MFMA, "unit": "TFLOP/s",
                          "frac": round(tf64 / PEAK_F64_MFMA, 4), "traffic": stored_traffic("traffic_bytes_per_launch_fp64"),
                          "instruction_loop_tflops_measured": MEASURED_F64_MFMA_LOOP,
                          "launches": len(k64), "avg_launch_ms": round(1e3 * t64 / max(len(k64), 1), 4),
                          "flops_per_launch": round(flops64 / max(len(k64), 1), 1)},
        "roofline_split_fp16": {"kernel": "gemm_bf16_grouped_kernel<float, float, 2, 2, fp16> (X updates and the root iterations "
                                          "after the fp64 prefix: fp32 operands split in two fp16 terms, 3 fp16 MFMA passes per product)",
                                "bound": "mfma", "achieved": round(3 * tf16, 2), "peak": PEAK_BF16_MFMA,
                                "unit": "TFLOP/s (fp16 MFMA issued)", "frac": round(3 * tf16 / PEAK_BF16_MFMA, 4),
                                "fp32_equivalent_tflops": round(tf16, 2),
                                "traffic": stored_traffic("traffic_bytes_per_launch_fp16"), "launches": len(k16),
                                "avg_launch_ms": round(1e3 * t16 / max(len(k16), 1), 4),
                                "flops_per_launch": round(3 * flops16 / max(len(k16), 1), 1)},
        "roofline_int8_slices": {"kernel": "gemm_i8_grouped_kernel<4 | 5 slices> (products of the fp64 iterations: each fp64 operand as its "
                                           "diagonal plus 7-bit slices, 10 | 15 int8 MFMA passes per product, exact int32 sums, fp64 assembly; "
                                           "the slice count is chosen per factor and product on the device)",
                                 "bound": "mfma", "achieved": round(tf8 * passes8, 2), "peak": PEAK_I8_MFMA,
                                 "unit": "TOP/s (int8 MFMA issued: lower bound, 10 passes per product)",
                                 "frac": round(tf8 * passes8 / PEAK_I8_MFMA, 4),
                                 "fp64_equivalent_tflops": round(tf8, 2),
                                 "traffic": stored_traffic("traffic_bytes_per_launch_int8"),
                                 "launches": len(k8), "avg_launch_ms": round(1e3 * t8 / max(len(k8), 1), 4),
                                 "flops_per_launch": round(flops8 * passes8 / max(len(k8), 1), 1)},
        "gemm_time_share_ms_per_step": {"fp32": round(1e3 * t32 / args.steps, 1), "fp64": round(1e3 * t64 / args.steps, 1),
                                        "split_fp16": round(1e3 * t16 / args.steps, 1), "int8_slices": round(1e3 * t8 / args.steps, 1)},
        "roofline_stats": {"bound": "hbm", "achieved": round(stats_bytes / stats_ms / 1e6, 1), "peak": PEAK_HBM,
                           "unit": "GB/s", "frac": round(stats_bytes / stats_ms / 1e6 / PEAK_HBM, 4),
                           "tflops": round(stats_flops / stats_ms / 1e9, 1)},
        # bf16 gradients: U^T = X_R G^T issues 2 bf16 MFMA passes (X_R split), P = X_L U issues 3 (both split)
        "roofline_precondition": {"bound": "mfma", "achieved": round(precond_issued / precond_ms / 1e9, 1),
                                  "peak": PEAK_BF16_MFMA, "unit": "TFLOP/s (bf16 MFMA issued)",
                                  "frac": round(precond_issued / precond_ms / 1e9 / PEAK_BF16_MFMA, 4),
                                  "fp32_equivalent_tflops": round(precond_flops / precond_ms / 1e9, 1),
                                  "gbps": round(precond_bytes / precond_ms / 1e6, 1)},
    }

    # `roofline` = the kernel that takes the largest share of the timed region
    shares = {"roofline_fp32": t32, "roofline_fp64": t64, "roofline_split_fp16": t16, "roofline_int8_slices": t8}
    if not k32:
        del out["roofline_fp32"], shares["roofline_fp32"]     # the default precision rules launch no fp32 product
    if not k8:
        del out["roofline_int8_slices"], shares["roofline_int8_slices"]
    elif on_i8:
        del out["roofline_fp64"], shares["roofline_fp64"]     # its launches were empty: every product passed the estimate
    dominant = max(shares, key=shares.get)
    out["roofline"] = dict(out[dominant], time_share_of_step=round(1e3 * shares[dominant] / args.steps / step_ms, 4))

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(fsize, Ls, Rs, shapes, eps_rel)
    if not args.no_soap:
        del blocks, factors, pblocks, Gs, Ls, Rs, XLs, XRs, Ps, ws
        torch.cuda.empty_cache()
        out["soap"] = soap_section(args, torch, ast, W, dev)
    print(json.dumps(out), flush=True)
    return 0


def soap_section(args, torch, ast, W, dev):
    """SOAP variant on the same model, blocks <= 2048 (318 blocks, 636 factors): three warm
    refreshes from Q = I, then `steps` x (soap_step + stats_update) and one eigenbasis refresh,
    each timed with events on the stream the library launches on."""
    beta, b1, b2, adam_eps = 0.95, 0.9, 0.95, 1e-8
    shapes = W.block_shapes(W.llama_1b_matrices(), 2048)
    if args.max_blocks:
        shapes = shapes[:: max(1, len(shapes) // args.max_blocks)][: args.max_blocks]
    bank = W.TemplateBank(dev)
    bases = [(bank.get(m, b), bank.get(n, b + 3)) for b, (m, n) in enumerate(shapes)]
    nsets = 2                                   # two gradient sets, used alternately
    Gsets = [[W.soap_gradient(U, V, t, dev, b) for b, (U, V) in enumerate(bases)] for t in range(nsets)]
    Ls = [torch.zeros(m, m, device=dev) for m, n in shapes]
    Rs = [torch.zeros(n, n, device=dev) for m, n in shapes]
    QLs = [torch.eye(m, device=dev) for m, n in shapes]
    QRs = [torch.eye(n, device=dev) for m, n in shapes]
    Ms = [torch.zeros(m, n, device=dev) for m, n in shapes]
    Vs = [torch.zeros(m, n, device=dev) for m, n in shapes]
    Ns = [torch.empty(m, n, device=dev) for m, n in shapes]
    blocks = [ast.Blocks(list(zip(G, Ls, Rs))) for G in Gsets]
    sblocks = [ast.SBlocks(list(zip(G, QLs, QRs, Ms, Vs, Ns))) for G in Gsets]
    factors = ast.Factors(list(zip(Ls, QLs)) + list(zip(Rs, QRs)))
    fsize = [m for m, n in shapes] + [n for m, n in shapes]
    need = max(ast.soap_refresh_workspace_bytes(factors)[0], ast.soap_step_workspace_bytes(sblocks[0]),
               ast.stats_update_workspace_bytes(blocks[0]))
    ws = torch.empty(int(need), dtype=torch.uint8, device=dev)
    info = torch.zeros(len(factors), dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    log(f"[bench] soap: {len(shapes)} blocks, {len(factors)} factors, workspace {need / 2**30:.1f} GiB, "
        f"{torch.cuda.memory_allocated() / 2**30:.1f} GiB resident")
    aux = [torch.cuda.Stream(), torch.cuda.Stream()]   # two groups of factors side by side (default priority)
    for w in range(3):                          # warm the bases from the identity
        ast.stats_update(blocks[w % nsets], beta, ws=ws)
        ast.soap_refresh(factors, info=info, ws=ws, aux_streams=aux)
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    for t in range(args.steps):
        ev[t][0].record()
        ast.soap_step(sblocks[t % nsets], b1, b2, adam_eps, t + 1, ws=ws)
        ev[t][1].record()
        ast.stats_update(blocks[t % nsets], beta, ws=ws)
        ev[t][2].record()
    r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    r0.record()
    ast.soap_refresh(factors, info=info, ws=ws, aux_streams=aux)
    r1.record()
    torch.cuda.synchronize()
    step_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / args.steps
    stats_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / args.steps
    refresh_ms = r0.elapsed_time(r1)
    # sanity of the refreshed bases (fp64 check of two factors, largest first, and of up to six
    # factors that the refresh reported as failed)
    def orth_of(Q):
        q = Q.double()
        return float(torch.linalg.norm(q.T @ q - torch.eye(q.shape[0], device=dev, dtype=torch.float64)) / q.shape[0] ** 0.5)
    allQ = QLs + QRs
    # ... plus the right factor of the first wide block (m < n / 4): its statistic has rank <= 5 m < n
    # after the five updates of this section, the case the refresh handles with a third sweep
    wide = [len(shapes) + b for b, (m, n) in enumerate(shapes) if 4 * m < n][:1]
    orth = max([orth_of(QLs[0]), orth_of(QRs[-1])] + [orth_of(allQ[i]) for i in wide])
    flagged = [i for i, v in enumerate(info.cpu().tolist()) if v != 0]
    orth_flagged = max([orth_of(allQ[i]) for i in flagged[:: max(1, len(flagged) // 6)][:6]], default=0.0)
    if flagged:
        log(f"[bench] soap: {len(flagged)} factors reported failed, sizes {sorted(set(fsize[i] for i in flagged))}, "
            f"orthogonality of a sample of them {orth_flagged:.1e}")
    step_flops = sum(2.0 * (2.0 * m * m * n + 2.0 * m * n * n) for m, n in shapes)
    step_issued = sum((2.0 + 3.0) * 2.0 * m * n * n + (3.0 + 3.0) * 2.0 * m * m * n for m, n in shapes)
    refresh_flops = sum((2.0 + 8.0 / 3.0) * float(n) ** 3 for n in fsize)
    adam_bytes = sum(24.0 * m * n for m, n in shapes)
    log(f"[bench] soap: step {step_ms:.1f} ms + stats {stats_ms:.1f} ms, refresh {refresh_ms:.1f} ms, "
        f"orthogonality {orth:.1e}, info!=0: {int((info != 0).sum())}")
    return {"workload": "same 1.1B model, blocks <=2048: 318 blocks, 636 factors; shared singular bases, "
                        "+-30% sigma jitter, 10% dense noise; beta1=0.9, beta2=0.95",
            "blocks": len(shapes), "factors": len(factors),
            "soap_step_ms": round(step_ms, 3), "stats_update_ms": round(stats_ms, 3),
            "refresh_ms": round(refresh_ms, 3),
            "amortised_step_pf10": round(step_ms + stats_ms + refresh_ms / 10, 3),
            "soap_step_tflops": round(step_flops / step_ms / 1e9, 1),
            # bf16 gradients: G Q_R issues 2 bf16 MFMA passes, the other three products 3 each (split operands)
            "soap_step_bf16_issued_tflops": round(step_issued / step_ms / 1e9, 1),
            "soap_step_frac_bf16_mfma": round(step_issued / step_ms / 1e9 / PEAK_BF16_MFMA, 4),
            "refresh_dense_tflops": round(refresh_flops / refresh_ms / 1e9, 1),
            "adam_bytes_gb": round(adam_bytes / 1e9, 2),
            "orthogonality_max": max(orth, orth_flagged), "not_ok": int((info != 0).sum())}


def cpu_baseline(fsize, Ls, Rs, shapes, eps_rel):
    """The float64 oracle (cyclic Jacobi + explicit spectral root), one factor per host thread, on
    a bounded sample of the same statistics; extrapolated to the full refresh by n^3."""
    import numpy as np
    import torch
    import oracle

    cores = min(16, os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16")))
    sample = [L for L, (m, n) in zip(Ls, shapes) if m == 512][:cores]
    if len(sample) < cores:
        sample += [R for R, (m, n) in zip(Rs, shapes) if n == 512][: cores - len(sample)]
    if not sample:                      # truncated debug batch: take the smallest factors
        sample = sorted(Ls + Rs, key=lambda t: t.shape[0])[:cores]
    As = [a.detach().to("cpu", torch.float32).double().numpy() for a in sample]
    os.environ["OMP_NUM_THREADS"] = str(cores)
    t = time.time()
    Xs, lmax, status = oracle.inverse_root_batch(As, eps_rel)
    dt = time.time() - t
    work_sample = sum(a.shape[0] ** 3 for a in As)
    work_full = sum(float(n) ** 3 for n in fsize)
    full_ms = 1e3 * dt * work_full / work_sample
    log(f"[bench] oracle: {len(As)} factors n={As[0].shape[0]} on {cores} threads in {dt:.1f} s "
        f"-> extrapolated full refresh {full_ms / 1e3:.0f} s")
    return {"value": round(full_ms, 1), "unit": "ms per full refresh (extrapolated by n^3 from the sample)",
            "cores": cores, "kind": "oracle", "measured_s": round(dt, 2),
            "sample": f"{len(As)} factors of n={As[0].shape[0]} from this workload's statistics, one per thread "
                      f"(cyclic-Jacobi float64 inverse 4th root), status ok: {int((status == 0).sum())}/{len(As)}"}


if __name__ == "__main__":
    sys.exit(main())
