"""The paper's 72-shape benchmark grid as synthetic inputs, on one MI355X.

    python -m paper_2311_00368_amd.sweep [--out sweep72.md] [--iters 10] [--bf16 | --plan]
    python -m paper_2311_00368_amd.sweep --skew [--out skew.md] [--iters 10]
    python -m paper_2311_00368_amd.sweep --three-way [--out threeway.md] [--iters 10]

The grid is the one on the x axes of the paper's benchmark figures: 12 (M, K) pairs x sparsity
70 / 80 / 90 % x N in {32, 128}, with D = N as in the paper.  The paper's own matrices (the
collection of [Trevor2020]) are randomized and not available; each point is a seeded Bernoulli
pattern of the same size and density with U[-1,1] values (`inputs.custom_workload`).  For every
point SPMM, SDDMM and FusedMM run `iters` times after two warm-ups; the time is the minimum over
the runs (the paper's protocol: minimum of 20 back-to-back runs) of the HIP-event pair the
library records around each call's kernels.  Gflop/s use 2*nnz*N, 2*nnz*D and 2*nnz*(D+N).

The output is a markdown table; the bars of the paper's figures (Intel Data Center GPU Max 1550,
one stack; other hardware, context only; `paper_grid_bars.txt`) are put next to the measured numbers.

--skew: uneven rows instead of the grid.  The pattern of the `fused8k_skew` workload (8192 x 8192, row lengths
log-normal with mean 10 % of K and sigma 1) with D = 64 and N in {64, 128, 256, 512}; SPMM and FusedMM, unplanned
and planned, microseconds per call (minimum), and the same calls with the LDS-tiled kernels switched off
(CSRK_KTILE=3: the equal-share kernels only) for comparison.

--three-way: every grid point and operation timed five times - automatic choice, the LDS-tiled kernels forced
(CSRK_KTILE=2), the whole-row kernels forced (CSRK_KTILE=3 CSRK_ROWS=2), equal shares forced (CSRK_KTILE=3
CSRK_ROWS=3), and a planned call - in microseconds per call (minimum), with the longest row of the pattern and the
families that csrk_explain_choice names for the point (unplanned and planned).  The table is what tests/test_dispatch_choice.py replays the choice against.
"""
from __future__ import annotations

import argparse
import os
import sys
import time

MK = [(1, 1), (3, 1), (4, 1), (2, 2), (6, 2), (8, 2), (4, 4), (12, 4), (16, 4), (8, 8), (24, 8), (32, 8)]
SPARSITY = [70, 80, 90]
WIDTHS = [32, 128]


def paper_bars():
    """{(Mk, Kk, sparsity): [sddmm32, sddmm128, spmm32, spmm128, fused32, fused128]}: the bars of the paper's
    benchmark figures (section "Performance results"), from the text file next to this module."""
    out = {}
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_grid_bars.txt")) as f:
        for line in f:
            cells = line.split("#")[0].split()
            if len(cells) == 9:
                out[(int(cells[0]), int(cells[1]), int(cells[2]))] = [int(c) for c in cells[3:]]
    return out


def skew_table(args, torch, binding, inputs):
    """Uneven rows: see the module text."""
    import numpy as np
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    w = inputs.workload("fused8k_skew")
    f = w.ops["fusedmm"]
    M, K, D = w.M, w.K, f["D"]
    rp, ci, v = dev(w.rowptr), dev(w.colidx), dev(w.vals)
    A, B = dev(f["A"]), dev(f["B"])
    lens = np.diff(w.rowptr)

    def best_us(fn):
        fn()
        fn()
        torch.cuda.synchronize()
        binding.csrk_profile_enable(args.iters)
        for _ in range(args.iters):
            fn()
        torch.cuda.synchronize()
        times = [ms for _, ms in binding.csrk_profile_collect(args.iters + 4)]
        binding.csrk_profile_enable(0)
        return min(times) * 1e3

    lines = []
    for n in (64, 128, 256, 512):
        C = dev(inputs.uniform(0, inputs.STREAM_C, (K, n)))
        O = torch.empty((M, n), dtype=torch.float32, device="cuda")
        cells = []
        for mode in ("1", "3"):             # automatic choice; LDS-tiled kernels off
            os.environ["CSRK_KTILE"] = mode
            plan = binding.csrk_plan_create(M, K, rp, ci)
            cells += [best_us(lambda: binding.spmm_csr(M, K, n, rp, ci, v, C, O)),
                      best_us(lambda: binding.spmm_csr_plan(plan, n, v, C, O)),
                      best_us(lambda: binding.fusedmm_csr(M, K, D, n, rp, ci, v, A, B, C, O)),
                      best_us(lambda: binding.fusedmm_csr_plan(plan, D, n, v, A, B, C, O))]
            binding.csrk_plan_destroy(plan)
        os.environ.pop("CSRK_KTILE", None)
        lines.append((n, cells))
        print(n, " ".join(f"{c:8.1f}" for c in cells), flush=True)
    os.makedirs(os.path.dirname(os.path.abspath(args.out)), exist_ok=True)
    with open(args.out, "w") as fo:
        fo.write(f"8192 x 8192, nnz = {w.nnz}, row lengths log-normal (mean {lens.mean():.0f}, longest {lens.max()}), D = 64; "
                 f"microseconds per call, minimum over {args.iters} runs.\n\n")
        fo.write("| N | SPMM | SPMM planned | FusedMM | FusedMM planned | equal shares only: SPMM | SPMM planned | FusedMM | FusedMM planned |\n")
        fo.write("|---|---|---|---|---|---|---|---|---|\n")
        for n, cells in lines:
            fo.write(f"| {n} | " + " | ".join(f"{c:.1f}" for c in cells) + " |\n")
    print(f"wrote {args.out}")


def three_way_table(args, torch, binding, inputs):
    """Automatic choice against each forced family: see the module text."""
    import numpy as np
    dev = lambda a: torch.from_numpy(a).cuda()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    modes = (("auto", {}), ("tiled", {"CSRK_KTILE": "2"}), ("rows", {"CSRK_KTILE": "3", "CSRK_ROWS": "2"}),
             ("shares", {"CSRK_KTILE": "3", "CSRK_ROWS": "3"}))
    points = [(mk, sp, n) for mk in MK for sp in SPARSITY for n in WIDTHS]
    if args.limit:
        points = points[: args.limit]
    lines = []
    for (mk, kk), sp, n in points:
        M, K, D = mk * 1024, kk * 1024, n
        w = inputs.custom_workload(M, K, 1.0 - sp / 100.0, n, D)
        nnz, longest = w.nnz, int(np.diff(w.rowptr).max())
        rp, ci, v = dev(w.rowptr), dev(w.colidx), dev(w.vals)
        A, B, C = dev(w.ops["fusedmm"]["A"]), dev(w.ops["fusedmm"]["B"]), dev(w.ops["fusedmm"]["C"])
        O = torch.empty((M, n), dtype=torch.float32, device="cuda")
        P = torch.empty((nnz,), dtype=torch.float32, device="cuda")
        calls = (("spmm", binding.CSRK_OP_SPMM, lambda: binding.spmm_csr(M, K, n, rp, ci, v, C, O)),
                 ("sddmm", binding.CSRK_OP_SDDMM, lambda: binding.sddmm_csr(M, K, D, rp, ci, v, A, B, P)),
                 ("fusedmm", binding.CSRK_OP_FUSEDMM, lambda: binding.fusedmm_csr(M, K, D, n, rp, ci, v, A, B, C, O)))
        plan = binding.csrk_plan_create(M, K, rp, ci)
        planned_calls = {"spmm": lambda: binding.spmm_csr_plan(plan, n, v, C, O),
                         "sddmm": lambda: binding.sddmm_csr_plan(plan, D, v, A, B, P),
                         "fusedmm": lambda: binding.fusedmm_csr_plan(plan, D, n, v, A, B, C, O)}
        for name, op, fn in calls:
            us = {}
            for mode, env in modes + (("planned", {}),):
                if mode == "planned":
                    fn = planned_calls[name]
                for k in ("CSRK_KTILE", "CSRK_ROWS"):
                    os.environ.pop(k, None)
                os.environ.update(env)
                fn()
                fn()
                torch.cuda.synchronize()
                binding.csrk_profile_enable(args.iters)
                for _ in range(args.iters):
                    fn()
                torch.cuda.synchronize()
                us[mode] = min(ms for _, ms in binding.csrk_profile_collect(args.iters + 4)) * 1e3
                binding.csrk_profile_enable(0)
            for k in ("CSRK_KTILE", "CSRK_ROWS"):
                os.environ.pop(k, None)
            fam = binding.csrk_explain_choice(op, cus, M, K, n, D, nnz, longest)
            famp = binding.csrk_explain_choice(op, cus, M, K, n, D, nnz, longest, planned=True)
            lines.append((f"{mk}k/{kk}k/{n}/{sp}%", M, K, n, nnz, longest, name, us, fam, famp))
            print(lines[-1][0], name, " ".join(f"{m} {t:8.1f}" for m, t in us.items()), binding.FAMILY_NAMES[fam], "/",
                  binding.FAMILY_NAMES[famp], flush=True)
        binding.csrk_plan_destroy(plan)
        del rp, ci, v, A, B, C, O, P
    os.makedirs(os.path.dirname(os.path.abspath(args.out)), exist_ok=True)
    with open(args.out, "w") as f:
        f.write(f"| shape | M | K | N = D | nnz | longest row | operation | automatic | tiled forced | whole rows forced | equal shares forced | planned | family named by csrk_explain_choice ({cus} CUs) | ... for a planned call |\n")
        f.write("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|\n")
        for shape, M, K, n, nnz, longest, name, us, fam, famp in lines:
            f.write(f"| {shape} | {M} | {K} | {n} | {nnz} | {longest} | {name} | {us['auto']:.1f} | {us['tiled']:.1f} | {us['rows']:.1f} | "
                    f"{us['shares']:.1f} | {us['planned']:.1f} | {binding.FAMILY_NAMES[fam]} | {binding.FAMILY_NAMES[famp]} |\n")
        f.write(f"\nMicroseconds per call (HIP-event pair around all kernels of a call), minimum over {args.iters} runs.\n")
    print(f"wrote {args.out}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default="sweep72.md")
    ap.add_argument("--iters", type=int, default=10)
    ap.add_argument("--limit", type=int, default=0, help="only the first LIMIT grid points (debug)")
    ap.add_argument("--bf16", action="store_true",
                    help="dense operands rounded to bfloat16 and the *_csr_bf16 entry points instead of the FP32 ones")
    ap.add_argument("--skew", action="store_true", help="uneven rows instead of the grid (see the module text)")
    ap.add_argument("--three-way", action="store_true", help="automatic choice against forced families (see the module text)")
    ap.add_argument("--plan", action="store_true",
                    help="the pattern analysed once per shape (csrk_plan_create) and the *_csr_plan entry points: the "
                         "caller that reuses a pattern, and the paper's own protocol, which times kernels only")
    args = ap.parse_args()
    if args.plan and args.bf16:
        sys.exit("--plan and --bf16 exclude each other (there are no planned bfloat16 calls)")

    import torch

    from . import binding, inputs

    if not torch.cuda.is_available():
        sys.exit("sweep needs a GPU")
    binding.load(build_if_missing=False)
    if args.skew:
        return skew_table(args, torch, binding, inputs)
    if args.three_way:
        return three_way_table(args, torch, binding, inputs)
    dev = lambda a: torch.from_numpy(a).cuda()
    bars = paper_bars()
    rows = []
    points = [(mk, sp, n) for mk in MK for sp in SPARSITY for n in WIDTHS]
    if args.limit:
        points = points[: args.limit]
    t_start = time.time()
    for (mk, kk), sp, n in points:
        M, K, D = mk * 1024, kk * 1024, n
        w = inputs.custom_workload(M, K, 1.0 - sp / 100.0, n, D)
        nnz = w.nnz
        rp, ci, v = dev(w.rowptr), dev(w.colidx), dev(w.vals)
        A, B, C = dev(w.ops["fusedmm"]["A"]), dev(w.ops["fusedmm"]["B"]), dev(w.ops["fusedmm"]["C"])
        O = torch.empty((M, n), dtype=torch.float32, device="cuda")
        P = torch.empty((nnz,), dtype=torch.float32, device="cuda")
        calls = {
            "sddmm": (lambda: binding.sddmm_csr(M, K, D, rp, ci, v, A, B, P), 2.0 * nnz * D),
            "spmm": (lambda: binding.spmm_csr(M, K, n, rp, ci, v, C, O), 2.0 * nnz * n),
            "fusedmm": (lambda: binding.fusedmm_csr(M, K, D, n, rp, ci, v, A, B, C, O), 2.0 * nnz * (D + n)),
        }
        if args.bf16:
            import numpy as np
            h = lambda a: torch.from_numpy(inputs.to_bf16(a)[0].view(np.int16)).cuda().view(torch.bfloat16)
            A16, B16, C16 = h(w.ops["fusedmm"]["A"]), h(w.ops["fusedmm"]["B"]), h(w.ops["fusedmm"]["C"])
            calls = {
                "sddmm": (lambda: binding.sddmm_csr_bf16(M, K, D, rp, ci, v, A16, B16, P), 2.0 * nnz * D),
                "spmm": (lambda: binding.spmm_csr_bf16(M, K, n, rp, ci, v, C16, O), 2.0 * nnz * n),
                "fusedmm": (lambda: binding.fusedmm_csr_bf16(M, K, D, n, rp, ci, v, A16, B16, C16, O), 2.0 * nnz * (D + n)),
            }
        plan = None
        if args.plan:
            plan = binding.csrk_plan_create(M, K, rp, ci)
            calls = {
                "sddmm": (lambda: binding.sddmm_csr_plan(plan, D, v, A, B, P), 2.0 * nnz * D),
                "spmm": (lambda: binding.spmm_csr_plan(plan, n, v, C, O), 2.0 * nnz * n),
                "fusedmm": (lambda: binding.fusedmm_csr_plan(plan, D, n, v, A, B, C, O), 2.0 * nnz * (D + n)),
            }
        res = {}
        for name, (fn, flops) in calls.items():
            fn()
            fn()
            torch.cuda.synchronize()
            binding.csrk_profile_enable(args.iters)
            for _ in range(args.iters):
                fn()
            torch.cuda.synchronize()
            times = [ms for _, ms in binding.csrk_profile_collect(args.iters + 4)]
            binding.csrk_profile_enable(0)
            res[name] = flops / min(times) / 1e6          # Gflop/s
        rows.append(((mk, kk, sp, n), nnz, res))
        print(f"{mk}k/{kk}k/{n}/{sp}%  nnz={nnz}  " + "  ".join(f"{k} {x:8.0f}" for k, x in res.items()), flush=True)
        if plan is not None:
            binding.csrk_plan_destroy(plan)
        del rp, ci, v, A, B, C, O, P
    wall = time.time() - t_start

    col = {"sddmm": 0, "spmm": 2, "fusedmm": 4}
    os.makedirs(os.path.dirname(os.path.abspath(args.out)), exist_ok=True)
    with open(args.out, "w") as f:
        f.write("| M/K/N/sparsity | nnz | SDDMM | SPMM | FusedMM | paper SDDMM | paper SPMM | paper FusedMM |\n")
        f.write("|---|---|---|---|---|---|---|---|\n")
        wins = total = 0
        for (mk, kk, sp, n), nnz, res in rows:
            pb = bars.get((mk, kk, sp))
            cells = []
            for name in ("sddmm", "spmm", "fusedmm"):
                if pb:
                    ref = pb[col[name] + (1 if n == 128 else 0)]
                    cells.append(str(ref))
                    total += 1
                    wins += res[name] > ref
                else:
                    cells.append("-")
            f.write(f"| {mk}k/{kk}k/{n}/{sp}% | {nnz} | {res['sddmm']:.0f} | {res['spmm']:.0f} | {res['fusedmm']:.0f} | "
                    + " | ".join(cells) + " |\n")
        f.write(f"\nGflop/s, minimum over {args.iters} runs per point; {len(rows)} grid points in {wall:.0f} s.\n")
        if total:
            f.write(f"Measured value above the paper's bar (Intel Max 1550, one stack; context, other hardware) in "
                    f"{wins} of {total} comparisons.\n")
    print(f"wrote {args.out}")


if __name__ == "__main__":
    main()
