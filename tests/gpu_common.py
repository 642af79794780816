"""Helpers for the GPU parity tests: run the HIP path through the C ABI binding and bring the
results back as numpy arrays shaped like the oracle's."""
import numpy as np
import torch

import paper_2405_10951_amd as P


def rel(a, b):
    """max|a-b| / max|b| per tensor (the tolerance the parity bar is stated in)."""
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    if b.size == 0:
        return 0.0
    return float(np.max(np.abs(a - b)) / max(float(np.max(np.abs(b))), 1e-30))


def bf16_rne(a):
    """fp32 -> the nearest bf16 value (ties to even), as fp32: what a bf16 copy of a weight matrix holds."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000).astype(np.uint32)
    return r.view(np.float32).reshape(np.shape(a))


def rel_rms(a, b):
    """rms(a-b) / rms(b)"""
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.sqrt(np.mean((a - b) ** 2)) / max(float(np.sqrt(np.mean(b ** 2))), 1e-30))


def outside_rate(a, b, rtol):
    """Fraction of elements with |a-b| > atol + rtol*|b|, atol = rtol * rms(b): the per-element form of the
    tolerance (a max-norm over ~10^5 elements is an extreme-value statistic, this is not)."""
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    atol = rtol * float(np.sqrt(np.mean(b ** 2)))
    return float(np.mean(np.abs(a - b) > atol + rtol * np.abs(b)))


def run_hip_step(cfg, params, x, labels, forced_idx=None, max_batch=None, sgd=None, ctx=None,
                 forced_experts=None, adamw=None, autotune=False):
    """One BSR step on cuda:0.  forced_idx: list per drop of [B,k] arrays (or None).
    forced_experts: dict block -> [rows,K] expert choice for the mixture-of-experts blocks (or None).
    sgd: None or dict(lr=, momentum=, weight_decay=, momenta=dict|None).
    adamw: None or dict(lr=, beta1=, beta2=, eps=, weight_decay=, step=, exp_avg=dict, exp_avg_sq=dict).
    autotune: run the measured tile choice first (as bench.py does during set-up).
    Returns a dict."""
    dev = torch.device("cuda:0")
    B = x.shape[0]
    own = ctx is None
    if own:
        ctx = P.Context(cfg, params, max_batch or B)
    act = ctx.act_dtype
    xin = torch.as_tensor(x).to(dev).to(act).contiguous()
    lab = torch.as_tensor(labels, dtype=torch.int32).to(dev)

    def cat_idx(which):
        if forced_idx is None or not which:
            return None
        return torch.as_tensor(np.concatenate([np.asarray(forced_idx[i], np.int32).reshape(-1) for i in which]),
                               dtype=torch.int32).to(dev)

    def bufs(which):
        nk = sum(B * ctx.keep_k[i] for i in which)
        ns = sum(B * ctx.n_in(i) for i in which)
        return (torch.full((max(nk, 4),), -1, dtype=torch.int32, device=dev),
                torch.zeros(max(ns, 4), dtype=torch.float32, device=dev))

    moe_rows = ctx.moe_rows(B)
    ex_out = rl_out = None
    if moe_rows:
        K, E = ctx.c.moe_top_k, ctx.c.n_experts
        total = sum(moe_rows.values())
        ex_out = torch.full((total * K,), -1, dtype=torch.int32, device=dev)
        rl_out = torch.zeros(total * E, dtype=torch.float32, device=dev)
        fex = None
        if forced_experts is not None:
            fex = torch.as_tensor(np.concatenate([np.asarray(forced_experts[l], np.int32).reshape(-1)
                                                  for l in sorted(moe_rows)]), dtype=torch.int32).to(dev)
        ctx.bsr_moe_routing_io(fex, ex_out, rl_out)
    kf, sf = bufs(ctx.frozen_drops)
    kt, st = bufs(ctx.train_drops)
    if autotune:
        x_t = torch.empty((B, ctx.T_f, cfg["dim"]), dtype=act, device=dev)
        ctx.bsr_autotune(xin, lab, x_t, torch.zeros(1, dtype=torch.float32, device=dev), ctx.new_grads())
    x_f = ctx.bsr_forward_frozen(xin, kept_idx_out=kf, scores_out=sf, forced_idx=cat_idx(ctx.frozen_drops))
    grads = ctx.new_grads()
    C = max(cfg["num_classes"], 1)
    logits = torch.zeros((B, C), dtype=torch.float32, device=dev)
    x_final = torch.zeros((B, ctx.T_last, cfg["dim"]), dtype=act, device=dev)
    loss = ctx.bsr_train_blocks_fwd_bwd(x_f, lab, grads, logits_out=logits, x_final_out=x_final,
                                        kept_idx_out=kt, scores_out=st, forced_idx=cat_idx(ctx.train_drops))
    new_params = None
    if sgd is not None:
        mom = sgd.get("momenta")
        ctx.bsr_sgd_step(grads, mom, sgd["lr"], sgd.get("momentum", 0.0), sgd.get("weight_decay", 0.0))
        new_params = {n: ctx.params[n].detach().cpu().numpy().copy() for n in ctx.trainable_names}
    if adamw is not None:
        ctx.bsr_adamw_step(grads, adamw["exp_avg"], adamw["exp_avg_sq"], adamw["lr"], adamw["beta1"],
                           adamw["beta2"], adamw["eps"], adamw["weight_decay"], adamw["step"])
        new_params = {n: ctx.params[n].detach().cpu().numpy().copy() for n in ctx.trainable_names}
    torch.cuda.synchronize()

    kept, scores = [None] * ctx.c.n_drop, [None] * ctx.c.n_drop
    for which, kb, sb in ((ctx.frozen_drops, kf, sf), (ctx.train_drops, kt, st)):
        o1 = o2 = 0
        for i in which:
            k, n = ctx.keep_k[i], ctx.n_in(i)
            kept[i] = kb[o1:o1 + B * k].cpu().numpy().reshape(B, k)
            scores[i] = sb[o2:o2 + B * n].cpu().numpy().reshape(B, n)
            o1 += B * k
            o2 += B * n
    out = dict(kept_idx=kept, scores=scores, x_trainable=x_f.float().cpu().numpy(),
               x_final=x_final.float().cpu().numpy(), logits=logits.cpu().numpy(),
               loss=float(loss[0].item()), grads={n: g.cpu().numpy() for n, g in grads.items()},
               new_params=new_params, keep_k=ctx.keep_k, ctx=ctx)
    if moe_rows:
        K, E = ctx.c.moe_top_k, ctx.c.n_experts
        out["experts"], out["router_logits"], o = {}, {}, 0
        for l in sorted(moe_rows):
            m = moe_rows[l]
            out["experts"][l] = ex_out[o * K:(o + m) * K].cpu().numpy().reshape(m, K)
            out["router_logits"][l] = rl_out[o * E:(o + m) * E].cpu().numpy().reshape(m, E)
            o += m
    return out


def gap_ok(scores_row, k, rel_gap):
    """True when the oracle's k-th and (k+1)-th largest scores are separated by more than rel_gap
    (relative to the k-th): only then is the kept set required to match exactly."""
    if k == 0 or k >= scores_row.size:
        return True
    s = np.sort(scores_row)[::-1]
    return (s[k - 1] - s[k]) > rel_gap * abs(s[k - 1])
