"""A PyTorch-CPU autograd composition of the BSR step from library primitives (F.layer_norm,
F.linear, F.scaled_dot_product_attention / softmax, F.gelu, F.cross_entropy, F.conv2d).  Test-only:
it pins the C oracle and is independent of both the oracle's code and the HIP library."""
import math

import torch
import torch.nn.functional as F


def moe_ffn(h2, w_router, w1, b1, w2, b2, K, experts=None):
    """Mixture-of-experts FFN on tokens h2 [M,D] from library primitives: torch.topk on the router
    logits (or the given expert choice), softmax over the selected logits, one dense FFN per expert
    on the tokens routed to it (index_select / index_add).  Returns (y [M,D], experts [M,K])."""
    logits = h2 @ w_router
    if experts is None:
        experts = torch.topk(logits, K, dim=-1).indices
    else:
        experts = torch.as_tensor(experts, dtype=torch.long)
    gates = torch.softmax(torch.gather(logits, 1, experts), dim=-1)
    y = torch.zeros_like(h2)
    for e in range(w1.shape[0]):
        tok, slot = torch.nonzero(experts == e, as_tuple=True)
        if tok.numel() == 0:
            continue
        he = h2.index_select(0, tok)
        ye = F.linear(F.gelu(F.linear(he, w1[e].t(), b1[e])), w2[e].t(), b2[e])
        y = y.index_add(0, tok, ye * gates[tok, slot][:, None])
    return y, experts


def run(cfg, params, x, labels, kept_idx, dtype=torch.float64, eps=1e-6, experts=None):
    """kept_idx: list per drop of [B,k] integer arrays (constants); experts: dict block -> [M,K] expert
    choice for mixture-of-experts blocks (constants; None: torch.topk).  Returns dict with loss,
    logits, x_final, grads (for trainable tensors), scores (per drop), x_trainable, dx_trainable."""
    P = {k: torch.tensor(v, dtype=dtype) for k, v in params.items()}
    ft, L, D, H = cfg["first_trainable"], cfg["depth"], cfg["dim"], cfg["heads"]
    d = D // H
    tb = cfg.get("trainable_blocks")
    for name, t in P.items():
        blk = int(name.split(".")[1]) if name.startswith("blocks.") else -1
        tr = name in ("lnf_g", "lnf_b", "w_head", "b_head") or (blk >= 0 and ((blk in tb) if tb else blk >= ft))
        t.requires_grad_(tr)
    x = torch.tensor(x, dtype=dtype)
    B = x.shape[0]
    if cfg["image_size"]:
        p = cfg["patch_size"]
        w = P["w_patch"].t().reshape(D, cfg["in_chans"], p, p)
        e = F.conv2d(x, w, P["b_patch"], stride=p).flatten(2).transpose(1, 2)
        x = torch.cat([P["cls"].expand(B, 1, D), e], dim=1) + P["pos"]
    drops = list(cfg["drop_blocks"])
    scores, di, x_tr = [], 0, None
    for l in range(L):
        if l == ft:
            x = x.detach().requires_grad_(True)
            x_tr = x
        g = lambda n: P[f"blocks.{l}.{n}"]
        T = x.shape[1]
        h = F.layer_norm(x, (D,), g("ln1_g"), g("ln1_b"), eps)
        qkv = F.linear(h, g("w_qkv").t(), g("b_qkv")).reshape(B, T, 3, H, d).permute(2, 0, 3, 1, 4)
        q, k, v = qkv[0], qkv[1], qkv[2]
        att = torch.softmax(q @ k.transpose(-1, -2) / math.sqrt(d), dim=-1)
        o = (att @ v).transpose(1, 2).reshape(B, T, D)
        x = x + F.linear(o, g("w_proj").t(), g("b_proj"))
        if di < len(drops) and drops[di] == l:
            scores.append(att[:, :, 0, 1:].mean(dim=1).detach().numpy())
            idx = torch.tensor(kept_idx[di], dtype=torch.long)
            full = torch.cat([torch.zeros(B, 1, dtype=torch.long), idx + 1], dim=1)
            xk = torch.gather(x, 1, full[:, :, None].expand(B, full.shape[1], D))
            if cfg.get("fuse_dropped") and idx.shape[1] < T - 1:
                # importance-weighted average of the dropped tokens, weights detached (constants)
                a = att[:, :, 0, 1:].mean(dim=1).detach()
                wts = a.scatter(1, idx, 0.0)
                wts = wts / wts.sum(dim=1, keepdim=True)
                fused = torch.einsum("bn,bnd->bd", wts, x[:, 1:])
                xk = torch.cat([xk, fused[:, None, :]], dim=1)
            x = xk
            di += 1
        h2 = F.layer_norm(x, (D,), g("ln2_g"), g("ln2_b"), eps)
        if l in cfg.get("moe_blocks", ()):
            y, _ = moe_ffn(h2.reshape(-1, D), g("w_router"), g("w_fc1"), g("b_fc1"), g("w_fc2"), g("b_fc2"),
                           cfg["moe_top_k"], None if experts is None else experts[l])
            x = x + y.reshape(x.shape)
        else:
            u = F.linear(h2, g("w_fc1").t(), g("b_fc1"))
            x = x + F.linear(F.gelu(u), g("w_fc2").t(), g("b_fc2"))
    if ft == L:
        x = x.detach().requires_grad_(True)
        x_tr = x
    logits = None
    if cfg["num_classes"]:
        z = F.layer_norm(x[:, 0], (D,), P["lnf_g"], P["lnf_b"], eps)
        logits = F.linear(z, P["w_head"].t(), P["b_head"])
        loss = F.cross_entropy(logits, torch.tensor(labels, dtype=torch.long))
    else:
        loss = (x * x).mean()
    loss.backward()
    grads = {n: t.grad.numpy() for n, t in P.items() if t.requires_grad and t.grad is not None}
    return dict(loss=float(loss), logits=None if logits is None else logits.detach().numpy(),
                x_final=x.detach().numpy(), grads=grads, scores=scores,
                x_trainable=x_tr.detach().numpy(), dx_trainable=x_tr.grad.numpy(),
                untouched=[n for n, t in P.items() if not t.requires_grad])
