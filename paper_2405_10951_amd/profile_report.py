"""Text summaries of rocprofv3 runs of bench.py, and the per-launch table of the step's GEMMs.

    python -m paper_2405_10951_amd.profile_report trace <kernel_trace.csv> [steps]
        per-kernel table (launches, microseconds per step, share) of the last `steps` steps of a
        `rocprofv3 --kernel-trace` run; a step starts at its patchify dispatch, what runs before the
        counted steps (tile tuning, warm-up) is set-up.
    python -m paper_2405_10951_amd.profile_report counters <counter_collection.csv> [steps]
        per kernel class, the average of every counter of a `rocprofv3 --pmc` run over the last `steps` steps;
        where the run holds them, the matrix-core utilisation by rocprofv3's own definition of MfmaUtil
        (SQ_VALU_MFMA_BUSY_CYCLES summed / (GRBM_GUI_ACTIVE per XCD x 1024 SIMDs)), the same busy cycles against
        SQ_BUSY_CYCLES, and, for the four TCC_EA0_RDREQ size counters, the bytes the L2 asked the fabric for.
    python -m paper_2405_10951_amd.profile_report shapes [--workload W] [--batch B] [--fetch f.csv --write w.csv --steps N]
        needs the GPU: tunes the tile shapes as bench.py does and prints, launch by launch, the product, the
        shape chosen, its measured time, TFLOP/s, % of the bf16 MFMA peak and the algorithmic bytes (operands
        and result once); with the two counter files of a --pmc FETCH_SIZE / WRITE_SIZE run of
        `bench.py --no-pipeline --calibrate-copy --no-sweep`, also the HBM-side bytes each launch moved.
"""
from __future__ import annotations

import collections
import csv
import re
import sys

PEAK_BF16_TFLOPS = 2500.0


def _short(name: str) -> str:
    name = re.sub(r"\(anonymous namespace\)::", "", name)
    return re.sub(r"^void ", "", name)


def _is_gemm(name: str) -> bool:
    return "gemm_nt_kernel" in name or "gemm_ntd_kernel" in name or "gemm_tn_kernel" in name


def trace(path: str, nsteps: int = 20) -> None:
    rows = list(csv.DictReader(open(path)))
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    starts = [i for i, r in enumerate(rows) if "patchify" in r["Kernel_Name"]]
    nsteps = min(nsteps, len(starts))
    sel = rows[starts[-nsteps]:]
    agg: dict = collections.OrderedDict()
    for r in sel:
        a = agg.setdefault(_short(r["Kernel_Name"]), [0, 0.0])
        a[0] += 1
        a[1] += (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
    tot = sum(a[1] for a in agg.values())
    gemm = sum(a[1] for n, a in agg.items() if _is_gemm(n))
    span = (int(sel[-1]["End_Timestamp"]) - int(sel[0]["Start_Timestamp"])) / 1e3
    print(f"# last {nsteps} steps: {len(sel)} dispatches ({len(sel) / nsteps:.1f} per step), kernel time "
          f"{tot / nsteps:.1f} us per step, span {span / nsteps:.1f} us per step")
    print(f"# GEMM launches (gemm_nt / gemm_ntd / gemm_tn kernels): {gemm / nsteps:.1f} us per step, summed durations")
    print(f"{'kernel':72s} {'per_step':>8s} {'us/step':>9s} {'avg_us':>8s} {'pct':>6s}")
    for n, (c, t) in sorted(agg.items(), key=lambda kv: -kv[1][1]):
        print(f"{n[:72]:72s} {c / nsteps:8.1f} {t / nsteps:9.1f} {t / c:8.1f} {100 * t / tot:6.2f}")


def _counter_rows(path: str):
    """(dispatch id, kernel name, {counter: value}) in dispatch order; values of one counter are summed over
    the hardware instances rocprofv3 lists separately."""
    per: dict = collections.OrderedDict()
    with open(path) as f:
        for r in csv.DictReader(f):
            d = per.setdefault(int(r["Dispatch_Id"]), [r["Kernel_Name"], collections.defaultdict(float)])
            d[1][r["Counter_Name"]] += float(r["Counter_Value"])
    return [(k, v[0], v[1]) for k, v in sorted(per.items())]


def counters(path: str, nsteps: int = 5) -> None:
    rows = _counter_rows(path)
    starts = [i for i, r in enumerate(rows) if "patchify" in r[1]]
    nsteps = min(nsteps, len(starts))
    sel = rows[starts[-nsteps]:] + [r for r in rows[:starts[-nsteps]] if "copybuffer" in r[1].lower()][-1:]

    def cls(n: str) -> str:
        if "gemm_ntd_kernel" in n:
            return "gemm_ntd (operands straight into LDS)"
        if _is_gemm(n):
            return "gemm_nt / gemm_tn (register-staged; fused launches carry a weight gradient)"
        if "attn_fwd" in n:
            return "attention forward"
        if "attn_bwd" in n:
            return "attention backward"
        if "copybuffer" in n.lower():
            return "plain device-to-device copy (256 MiB read, 256 MiB written, when bench.py ran with --calibrate-copy)"
        return "other"

    agg: dict = collections.OrderedDict()
    for _, n, c in sel:
        a = agg.setdefault(cls(n), [0, collections.defaultdict(float)])
        a[0] += 1
        for k, v in c.items():
            a[1][k] += v
    names = sorted({k for a in agg.values() for k in a[1]})
    print(f"# last {nsteps} steps, {len(sel)} dispatches; counter averages per dispatch of a class")
    for c, (cnt, vals) in agg.items():
        print(f"{c}: {cnt / nsteps:.1f} launches per step")
        for k in names:
            print(f"    {k:36s} {vals[k] / cnt:16.1f}")
        if "SQ_VALU_MFMA_BUSY_CYCLES" in vals and vals.get("GRBM_GUI_ACTIVE", 0) > 0:
            # rocprofv3's MfmaUtil: busy cycles summed over all SIMDs / (active clocks of one XCD x 1024 SIMDs);
            # the values here are sums over the 8 XCDs, so the mean over XCDs stands for the maximum
            print(f"    {'MfmaUtil (busy / GUI active x 1024)':36s} "
                  f"{100.0 * vals['SQ_VALU_MFMA_BUSY_CYCLES'] / 1024.0 / (vals['GRBM_GUI_ACTIVE'] / 8.0):15.1f}%")
        if "SQ_VALU_MFMA_BUSY_CYCLES" in vals and "SQ_BUSY_CYCLES" in vals and vals["SQ_BUSY_CYCLES"] > 0:
            # both are summed over the shader engines; SQ_BUSY_CYCLES counts per SE, MFMA busy per SIMD:
            # 256 CUs x 4 SIMDs = 1024 SIMDs over 32 SEs
            print(f"    {'MFMA busy / SQ busy (per SIMD)':36s} "
                  f"{100.0 * vals['SQ_VALU_MFMA_BUSY_CYCLES'] / 1024.0 / (vals['SQ_BUSY_CYCLES'] / 32.0):15.1f}%")
        if "SQ_INSTS_VALU_MFMA_MOPS_BF16" in vals:
            print(f"    {'MFMA flop (MOPS_BF16 x 512)':36s} {vals['SQ_INSTS_VALU_MFMA_MOPS_BF16'] * 512 / cnt / 1e9:14.2f} G")
        if "TCC_EA0_RDREQ_sum" in vals:
            n32, n64, n128 = (vals.get(f"TCC_EA0_RDREQ_{b}B_sum", 0.0) for b in (32, 64, 128))
            rest = vals["TCC_EA0_RDREQ_sum"] - n32 - n64 - n128
            print(f"    {'read requests 32B/64B/128B/other':36s} {n32 / cnt:.0f} / {n64 / cnt:.0f} / {n128 / cnt:.0f} / {rest / cnt:.0f}")
            print(f"    {'bytes asked of the fabric (reads)':36s} {(32 * n32 + 64 * n64 + 128 * n128 + 64 * rest) / cnt / 1e6:14.1f} MB")
        if "SQ_LDS_BANK_CONFLICT" in vals and vals.get("SQ_LDS_IDX_ACTIVE", 0) > 0:
            print(f"    {'LDS bank-conflict cycles / active':36s} "
                  f"{100.0 * vals['SQ_LDS_BANK_CONFLICT'] / vals['SQ_LDS_IDX_ACTIVE']:15.1f}%")


def shapes(argv: list[str]) -> None:
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="c3_vit_b")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--steps", type=int, default=7)
    a = ap.parse_args(argv)
    import torch
    import bsr_synth as S
    import paper_2405_10951_amd as P
    cfg = S.get_config(a.workload)
    batch = a.batch or cfg["batch"]
    cfg["batch"] = batch
    ctx = P.Context(cfg, S.make_params(cfg), batch)
    x, y = S.make_inputs(cfg, batch=batch)
    dev = ctx.device
    xin = torch.as_tensor(x).to(dev).to(ctx.act_dtype).contiguous()
    lab = torch.as_tensor(y, dtype=torch.int32).to(dev)
    xf = torch.empty((batch, ctx.T_f, cfg["dim"]), dtype=ctx.act_dtype, device=dev)
    ctx.bsr_autotune(xin, lab, xf, torch.zeros(4, device=dev), ctx.new_grads())
    launches = [(0,) + t for t in ctx.bsr_tile_choices(0)] + [(1,) + t for t in ctx.bsr_tile_choices(1)]
    hbm = None
    if a.fetch and a.write:
        from .traffic import COPY_BYTES
        per = []
        for path, counter in ((a.fetch, "FETCH_SIZE"), (a.write, "WRITE_SIZE")):
            rows = [(d, n, c.get(counter, 0.0)) for d, n, c in _counter_rows(path)]
            starts = [i for i, r in enumerate(rows) if "patchify" in r[1]]
            ns = min(a.steps, len(starts))
            copy = max(v for _, n, v in rows if "copybuffer" in n.lower())
            scale = COPY_BYTES / copy
            acc = None
            for s in range(ns):
                lo = starts[-ns + s]
                hi = starts[-ns + s + 1] if s + 1 < ns else len(rows)
                g = []          # a weight gradient launched on its own counts with the input gradient before it
                for _, n, v in rows[lo:hi]:
                    if "gemm_tn_kernel" in n and g:
                        g[-1] += v * scale
                    elif _is_gemm(n):
                        g.append(v * scale)
                acc = g if acc is None else [p + q for p, q in zip(acc, g)]
            per.append([v / ns for v in acc])
        hbm = list(zip(*per))
    # a backward launch of a trained layer also carries that layer's weight gradient (same flops again)
    print(f"# {a.workload} batch {batch}: GEMM launches of one step in launch order (part 0: frozen prefix, 1: trainable part)")
    if hbm:
        print("# fetch / write: FETCH_SIZE and WRITE_SIZE of the launch, each scaled by what it reads for the 256 MiB copy; they")
        print("# count what the L2s exchange with the fabric (the 256 MB last-level cache sits behind it), split-K partial sums included;")
        print("# ratio = (fetch + write) / algorithmic bytes")
    print("# us: the chosen shape timed at that launch by bsr_autotune (HIP events, launch gap included); a trainable-part launch")
    print("# after the head (backward) carries the input gradient shown AND the weight gradient of its layer: TF counts both")
    hdr = f"{'part':>4s} {'rows':>6s} {'out':>5s} {'in':>5s} {'tile':>8s} {'us':>7s} {'TFLOP/s':>8s} {'%peak':>6s} {'alg MB':>7s}"
    print(hdr + (f" {'fetch MB':>8s} {'write MB':>8s} {'ratio':>6s}" if hbm else ""))
    tot_us = tot_fl = 0.0
    seen_fwd = 0
    n_fwd_train = 4 * (cfg["depth"] - cfg["first_trainable"]) if not cfg.get("moe_blocks") else None
    for i, (part, m, n, k, tile, us) in enumerate(launches):
        fl = 2.0 * m * n * k
        alg = 2.0 * (m * k + n * k + m * n)
        bwd = part == 1 and n_fwd_train is not None and seen_fwd >= n_fwd_train
        if part == 1:
            seen_fwd += 1
        if bwd:
            fl *= 2.0
            alg += 2.0 * (m * n + m * k) + 4.0 * n * k     # the weight gradient reads x and dy again, writes dW fp32
        tot_us += us
        tot_fl += fl
        line = (f"{part:4d} {m:6d} {n:5d} {k:5d} {tile:8d} {us:7.1f} {fl / us / 1e6 if us else 0:8.0f} "
                f"{100 * fl / us / 1e6 / PEAK_BF16_TFLOPS if us else 0:6.1f} {alg / 1e6:7.1f}")
        if hbm and i < len(hbm):
            line += f" {hbm[i][0] / 1e6:8.1f} {hbm[i][1] / 1e6:8.1f} {sum(hbm[i]) / alg:6.2f}"
        print(line)
    print(f"# sum: {tot_us:.1f} us, {tot_fl / 1e9:.1f} GFLOP, {tot_fl / tot_us / 1e6:.0f} TFLOP/s "
          f"({100 * tot_fl / tot_us / 1e6 / PEAK_BF16_TFLOPS:.1f} % of the bf16 MFMA peak)")


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "trace":
        trace(sys.argv[2], int(sys.argv[3]) if len(sys.argv) > 3 else 20)
    elif len(sys.argv) >= 3 and sys.argv[1] == "counters":
        counters(sys.argv[2], int(sys.argv[3]) if len(sys.argv) > 3 else 5)
    elif len(sys.argv) >= 2 and sys.argv[1] == "shapes":
        shapes(sys.argv[2:])
    else:
        sys.exit(__doc__)
