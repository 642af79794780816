#!/usr/bin/env python3
"""Benchmark of the BSR fine-tuning step on one MI355X.

One "step" = bsr_forward_frozen -> bsr_train_blocks_fwd_bwd -> bsr_sgd_step on one batch of synthetic
ViT-B/16-shaped inputs already resident in HBM.  The timed steps are pipelined over two streams (the frozen
forward of the next batch beside the training part of the current one); the same steps run one after the
other are timed too and reported next to it.  Prints ONE JSON line: images/sec, the roofline of
the dominant kernel class (the bf16 MFMA GEMMs) and the CPU oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3


def build_context(cfg, batch, seed=0):
    import bsr_synth as S
    import paper_2405_10951_amd as P
    params = S.make_params(cfg, seed=seed)
    ctx = P.Context(cfg, params, batch)
    return ctx


def time_steps(ctx, cfg, batch, steps, warmup, profile_steps=0, autotune=True, pipeline=True):
    """Times `steps` steps one after the other on one stream and (when the model has a frozen prefix) pipelined:
    the frozen forward of batch i+1 on a second stream beside the training part and the optimizer step of
    batch i, with the tile shapes chosen launch by launch and again with the shape chosen for two streams.
    The frozen prefix reads frozen weights only, so all schedules compute the same thing; the fastest is the
    headline, the sequential figures are reported beside it."""
    import torch
    import bsr_synth as S
    dev = ctx.device
    x, y = S.make_inputs(cfg, batch=batch)
    xin = torch.as_tensor(x).to(dev).to(ctx.act_dtype).contiguous()
    lab = torch.as_tensor(y, dtype=torch.int32).to(dev)
    grads = ctx.new_grads()
    mom = {n: torch.zeros_like(g) for n, g in grads.items()}
    x_f = [torch.empty((batch, ctx.T_f, cfg["dim"]), dtype=ctx.act_dtype, device=dev) for _ in range(2)]
    loss = torch.zeros(4, dtype=torch.float32, device=dev)
    tuned = ctx.bsr_autotune(xin, lab, x_f[0], loss, grads) if autotune else None      # set-up, untimed

    def train(xf):
        ctx.bsr_train_blocks_fwd_bwd(xf, lab, grads, loss_out=loss)
        ctx.bsr_sgd_step(grads, mom, lr=1e-3, momentum=0.9, weight_decay=1e-4)

    def run_sequential(n):
        for _ in range(n):
            ctx.bsr_forward_frozen(xin, x_out=x_f[0])
            train(x_f[0])

    s_frozen, s_train = torch.cuda.Stream(), torch.cuda.Stream()

    def run_pipelined(n):
        cur = torch.cuda.current_stream()
        s_frozen.wait_stream(cur)
        s_train.wait_stream(cur)
        step = lambda inp, xn, xc: ctx.bsr_pipeline_step(inp, xn, xc, lab, loss, grads, mom, 1e-3, 0.9, 1e-4, s_frozen, s_train)
        step(xin, x_f[0], None)                                    # prime: the frozen prefix of batch 0
        for i in range(n):
            last = i + 1 == n
            step(None if last else xin, None if last else x_f[(i + 1) % 2], x_f[i % 2])
        cur.wait_stream(s_frozen)
        cur.wait_stream(s_train)

    def timed(run):
        run(warmup)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        run(steps)
        e1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return dict(wall_s=wall, ms_per_step=1e3 * wall / steps, ms_per_step_events=e0.elapsed_time(e1) / steps)

    def bracketed(run):        # per-launch event brackets of the GEMM / attention launches over profile_steps steps
        ctx.bsr_profile_begin()
        run(profile_steps)
        torch.cuda.synchronize()
        prof = ctx.bsr_profile_end()
        return {k: (v[0] / profile_steps, v[1] / profile_steps, v[2] // profile_steps) for k, v in prof.items()}

    def per_call(n):           # the three calls of a sequential step apart, and the spread of the step time
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(n)]
        for e in ev:
            e[0].record()
            ctx.bsr_forward_frozen(xin, x_out=x_f[0])
            e[1].record()
            ctx.bsr_train_blocks_fwd_bwd(x_f[0], lab, grads, loss_out=loss)
            e[2].record()
            ctx.bsr_sgd_step(grads, mom, lr=1e-3, momentum=0.9, weight_decay=1e-4)
            e[3].record()
        torch.cuda.synchronize()
        parts = [[e[i].elapsed_time(e[i + 1]) for e in ev] for i in range(3)]
        whole = sorted(ev[i][0].elapsed_time(ev[i + 1][0]) for i in range(n - 1))    # start to start
        med = lambda v: sorted(v)[len(v) // 2]
        return {"bsr_forward_frozen_ms": med(parts[0]), "bsr_train_blocks_fwd_bwd_ms": med(parts[1]),
                "bsr_sgd_step_ms": med(parts[2]), "step_ms_median": whole[len(whole) // 2], "step_ms_min": whole[0],
                "steps": n, "note": "HIP events between the calls of sequential steps, medians; taken after the timed region"}

    seq = timed(run_sequential)
    prof_seq = bracketed(run_sequential) if profile_steps else None
    calls = per_call(max(steps // 2, 10))
    has_prefix = (cfg.get("trainable_blocks") or [cfg["first_trainable"]])[0] > 0
    best, tuned_overlapped, tiles, prof_best = seq, None, "chosen launch by launch, each timed alone", prof_seq
    if pipeline and has_prefix:
        piped = timed(run_pipelined)                   # with the tile shapes chosen above
        if piped["ms_per_step"] < best["ms_per_step"]:
            best = piped
            prof_best = bracketed(run_pipelined) if profile_steps else None
        if autotune:           # tile shapes chosen again, now with the two parts of the step side by side
            torch.cuda.synchronize()
            with torch.cuda.stream(s_frozen):
                tuned_overlapped = ctx.bsr_autotune_overlapped(xin, lab, x_f[0], x_f[1], loss, grads, s_train)
            torch.cuda.synchronize()
            piped2 = timed(run_pipelined)
            if piped2["ms_per_step"] < best["ms_per_step"]:
                best, tiles = piped2, "one shape for every launch, chosen by timing the two parts side by side"
                prof_best = bracketed(run_pipelined) if profile_steps else None
    return dict(best, pipelined=best is not seq, tiles=tiles, sequential=seq, calls=calls, loss=float(loss[0].item()), prof=prof_best,
                prof_sequential=prof_seq, tuned=tuned, tuned_overlapped=tuned_overlapped)


def cpu_baseline(cfg, sample_batch, one_thread=True):
    """The oracle as it stands (float build, OpenMP over images), one full step of the same workload on all host
    cores, and once more on a single thread (in a child process: the thread count is fixed when OpenMP starts)."""
    import subprocess
    import bsr_synth as S
    from oracle import Oracle
    orc = Oracle("f32")
    p = S.make_params(cfg)
    x, y = S.make_inputs(cfg, batch=sample_batch)
    t0 = time.perf_counter()
    r = orc.step(cfg, p, x, y)
    dt = time.perf_counter() - t0
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    out = dict(value=sample_batch / dt, unit="images/sec", cores=cores, kind="oracle",
               sample=f"one full step (frozen forward, selection, trainable fwd+bwd) of the same workload on "
                      f"{sample_batch} of the {cfg['batch']} images, fp32 C oracle with OpenMP, {dt:.1f} s", loss=r["loss"])
    if one_thread:
        code = ("import sys, time, json; sys.path.insert(0, %r); import bsr_synth as S; from oracle import Oracle\n"
                "cfg = json.loads(sys.argv[1]); n = int(sys.argv[2]); orc = Oracle('f32'); p = S.make_params(cfg)\n"
                "x, y = S.make_inputs(cfg, batch=n); t0 = time.perf_counter(); orc.step(cfg, p, x, y)\n"
                "print(time.perf_counter() - t0)" % ROOT)
        n1 = sample_batch                           # (about 20 s for the 32 images of the headline workload)
        env = dict(os.environ, OMP_NUM_THREADS="1")
        try:
            res = subprocess.run([sys.executable, "-c", code, json.dumps(cfg), str(n1)], env=env, capture_output=True,
                                 text=True, timeout=300)
            dt1 = float(res.stdout.strip().splitlines()[-1])
            out["one_thread"] = dict(value=n1 / dt1, unit="images/sec", cores=1,
                                     sample=f"the same step on {n1} images, one thread, {dt1:.1f} s")
        except Exception as e:      # noqa: BLE001  (the baseline is context, never a reason to lose the line)
            out["one_thread"] = dict(value=None, error=str(e)[:200])
    return out


def recorded_traffic(workload, batch):
    """HBM bytes per GEMM launch from the committed rocprofv3 counter runs (profiles/gemm_traffic.json), or None
    when there is no record for this workload and batch or the GEMM source has changed since it was taken."""
    import hashlib
    rec = os.path.join(ROOT, "profiles", "gemm_traffic.json")
    src = os.path.join(ROOT, "paper_2405_10951_amd", "csrc", "k_gemm_mfma.hip")
    try:
        with open(rec) as f:
            d = json.load(f)
        with open(src, "rb") as f:
            sha = hashlib.sha256(f.read()).hexdigest()
        e = d.get("records", {}).get(f"{workload}/batch{batch}")
        if not e or e.get("kernel_source_sha256") != sha:
            return None
        return e["hbm_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def sweep_c4(P, S, step_flops_of, steps, warmup):
    """The shape sweep of the ablation tables at batch 128: keep ratio x number of trained blocks, one step after
    the other on one stream (with every block trained there is no frozen prefix to run ahead)."""
    import torch
    points = []
    for keep in (1.0, 0.7, 0.5):
        for trainable in (12, 4, 2):
            cfg = S.get_config("c3_vit_b", batch=128, keep_ratio=keep, first_trainable=12 - trainable)
            ctx = build_context(cfg, 128)
            r = time_steps(ctx, cfg, 128, steps, warmup, profile_steps=min(steps, 3), autotune=True, pipeline=False)
            fl = step_flops_of(cfg, ctx, 128)
            gemm_ms, gemm_flops, _ = r["prof"]["gemm"]
            points.append({"keep_ratio": keep, "trainable_blocks": trainable, "ms_per_step": r["ms_per_step"],
                           "images_per_sec": 128 * steps / r["wall_s"], "step_gflop": fl["total"] / 1e9,
                           "step_pct_of_bf16_mfma_peak": 100.0 * fl["total"] / (r["ms_per_step"] * 1e-3) / (PEAK_BF16_TFLOPS * 1e12),
                           "gemm_tflops_event_bracketed": gemm_flops / (gemm_ms * 1e-3) / 1e12})
            del ctx
            torch.cuda.empty_cache()
    return points


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c3_vit_b")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--keep-ratio", type=float, default=None)
    ap.add_argument("--trainable", type=int, default=None, help="number of trainable blocks (suffix)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-autotune", action="store_true", help="keep the cost model's tile choices")
    ap.add_argument("--no-compare", action="store_true", help="skip the keep-1.0 / full-fine-tuning legs")
    ap.add_argument("--no-pipeline", action="store_true",
                    help="time the steps one after the other only (no overlap of the next batch's frozen forward)")
    ap.add_argument("--cpu-sample", type=int, default=None, help="images of the cpu_baseline leg (default: the whole batch)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the batch-128 sweep keep ratio x trained blocks")
    ap.add_argument("--sweep", choices=["c4", "none"], default=None,
                    help="c4: the batch-128 sweep keep ratio {1.0, 0.7, 0.5} x trained blocks {12, 4, 2} under the `sweep` key "
                         "(the default on the headline workload at batch 32; with this flag on any ViT-B run); none: skip it")
    ap.add_argument("--sweep-steps", type=int, default=5)
    ap.add_argument("--fold-frozen-layernorm", action="store_true",
                    help="bsr_config.fold_frozen_layernorm = 1: the frozen prefix's LayerNorms ride inside the qkv / fc1 products")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures ONE GPU; --gpus must be 1 (no multi-GPU path exists)")

    import torch
    import bsr_synth as S
    import paper_2405_10951_amd as P
    from paper_2405_10951_amd.flops import step_flops
    if not torch.cuda.is_available():
        sys.exit("bench.py needs an MI355X (no CPU fallback exists)")
    P.load_library()

    cfg = S.get_config(args.workload)
    if args.keep_ratio is not None:
        cfg["keep_ratio"] = args.keep_ratio
    if args.trainable is not None:
        cfg["first_trainable"] = cfg["depth"] - args.trainable
    if args.fold_frozen_layernorm:
        cfg["fold_frozen_layernorm"] = 1
    batch = args.batch or cfg["batch"]
    cfg["batch"] = batch

    def flops_of(c, ctx, nb=None):
        pd = c["in_chans"] * c["patch_size"] ** 2
        return step_flops(c["dim"], c["mlp_hidden"], c["num_classes"], pd, ctx.tokens_attn[0] - 1,
                          ctx.tokens_attn, ctx.tokens_mlp, c["first_trainable"], nb or batch,
                          moe_blocks=tuple(c.get("moe_blocks", ())), n_experts=c.get("n_experts", 0),
                          moe_top_k=c.get("moe_top_k", 0), trainable_blocks=c.get("trainable_blocks"))

    ctx = build_context(cfg, batch)
    r = time_steps(ctx, cfg, batch, args.steps, args.warmup, profile_steps=min(args.steps, 10),
                   autotune=not args.no_autotune, pipeline=not args.no_pipeline)
    fl = flops_of(cfg, ctx)
    ips = batch * args.steps / r["wall_s"]
    bf16 = cfg["dtype"] == "bf16"
    peak = PEAK_BF16_TFLOPS if bf16 else PEAK_FP32_TFLOPS

    def roof(prof, schedule):
        """The GEMM launches of a step as one kernel class: flops launched / summed launch durations (HIP events
        recorded by the library around every launch, on the stream it is launched on)."""
        gemm_ms, gemm_flops, gemm_n = prof["gemm"]
        achieved = gemm_flops / (gemm_ms * 1e-3) / 1e12
        return {"bound": "mfma", "kernel": "GEMM launches of the step (forward, dgrad, wgrad)", "schedule": schedule,
                "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak, "traffic": None,
                "launches_per_step": gemm_n, "ms_per_step": gemm_ms, "gflop_per_step": gemm_flops / 1e9}

    sched_best = "pipelined (two streams)" if r["pipelined"] else "sequential (one stream)"
    out = {
        "metric": "BSR train images/sec, ViT-B/16 bs32 on 1 MI355X; % bf16 MFMA peak",
        "value": ips, "unit": "images/sec", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": f"{args.workload}: ViT dim {cfg['dim']} depth {cfg['depth']} batch {batch}, "
                               f"keep {cfg['keep_ratio']} at blocks {cfg['drop_blocks']}, "
                               + (f"trainable blocks {cfg['trainable_blocks']} + head, " if cfg.get("trainable_blocks")
                                  else f"trainable blocks {cfg['first_trainable']}..{cfg['depth'] - 1} + head, ")
                               + (f"{cfg['n_experts']}-expert top-{cfg['moe_top_k']} FFN in blocks {cfg['moe_blocks']}, "
                                  if cfg.get("moe_blocks") else "")
                               + "SGD momentum 0.9",
                   "global_batch": batch, "tokens_per_block": ctx.tokens_attn},
        "step_gflop": fl["total"] / 1e9,
        "step_pct_of_bf16_mfma_peak": 100.0 * fl["total"] / (r["ms_per_step"] * 1e-3) / (peak * 1e12),
        "ms_per_step_hip_events": r["ms_per_step_events"],
        "schedule": ("pipelined: the frozen forward of batch i+1 runs on a second stream beside the trainable part and "
                     "the optimizer step of batch i (frozen weights only, same results)") if r["pipelined"]
                    else "sequential: one step after the other on one stream",
        "tile_shapes": r["tiles"],
        "ms_per_step_sequential": r["sequential"]["ms_per_step"],
        "images_per_sec_sequential": batch * args.steps / r["sequential"]["wall_s"],
        "calls_sequential": r["calls"],
        "loss": r["loss"],
        "tile_autotune": None if r["tuned"] is None else {"launches": r["tuned"][0], "differ_from_cost_model": r["tuned"][1]},
        "tile_autotune_overlapped": None if r["tuned_overlapped"] is None else
        {"launches": r["tuned_overlapped"][0], "differ_from_cost_model": r["tuned_overlapped"][1]},
        # the roofline of the schedule that produced `value`; beside it the same figure for one step after the
        # other on one stream, where a launch has the GPU to itself (side by side, launches stretch each other)
        "roofline": roof(r["prof"], sched_best),
        "roofline_sequential": roof(r["prof_sequential"], "sequential (one stream)"),
        "kernel_classes_ms_per_step": {k: v[0] for k, v in r["prof"].items()},
    }
    out["roofline_sequential"]["traffic"] = recorded_traffic(args.workload, batch)
    if not r["pipelined"]:
        out["roofline"]["traffic"] = out["roofline_sequential"]["traffic"]
    else:
        # side by side a launch's bracket also holds the time it waits for, and shares the CUs with, the other stream's
        # launches, and the brackets of the two streams overlap: their sum exceeds the step.  The same flops over the
        # step's own wall time is what the matrix cores did for this class at the very least.
        over_wall = out["roofline"]["gflop_per_step"] / r["ms_per_step"]          # GFLOP / ms = TFLOP/s
        out["roofline"]["achieved_over_step_wall"] = over_wall
        out["roofline"]["frac_over_step_wall"] = over_wall / peak
    if args.calibrate_copy:
        a = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)                      # 256 MiB read + 256 MiB written by one elementwise copy kernel
        torch.cuda.synchronize()
        del a, b
    del ctx
    if not args.no_compare:
        cmp_steps = max(5, args.steps // 5)
        for key, over in (("speedup_vs_keep_1.0", dict(keep_ratio=1.0)),
                          ("speedup_vs_full_finetune", dict(keep_ratio=1.0, first_trainable=0))):
            c2 = dict(cfg, **over)
            ctx2 = build_context(c2, batch)
            r2 = time_steps(ctx2, c2, batch, cmp_steps, max(2, args.warmup // 2), pipeline=not args.no_pipeline)
            out[key] = r2["ms_per_step"] / r["ms_per_step"]                 # each side in its faster schedule
            out[key + "_sequential"] = r2["sequential"]["ms_per_step"] / r["sequential"]["ms_per_step"]
            out[key + "_algorithmic"] = flops_of(c2, ctx2)["total"] / fl["total"]
            del ctx2
            torch.cuda.empty_cache()
    want_sweep = args.sweep == "c4" or (args.sweep is None and not args.no_sweep and batch == 32)
    if want_sweep and args.workload == "c3_vit_b":
        out["sweep"] = {"workload": "c3_vit_b at batch 128, keep ratio x trained blocks (suffix), sequential schedule",
                        "points": sweep_c4(P, S, flops_of, args.sweep_steps, 2)}
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg, min(args.cpu_sample or batch, batch))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
