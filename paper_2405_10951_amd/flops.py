"""Algorithmic floating-point operations of one BSR step (2 x multiply-accumulates on the reduced
token sets the method actually processes; Sec. 4.3 Discussion 3 for the token counts).  Used by the
benchmark to turn a step time into a fraction of the MFMA roofline."""
from __future__ import annotations


def step_flops(dim: int, mlp_hidden: int, num_classes: int, patch_dim: int, n_patches: int,
               tokens_attn: list[int], tokens_mlp: list[int], first_trainable: int, batch: int,
               moe_blocks=(), n_experts: int = 0, moe_top_k: int = 0, trainable_blocks=None) -> dict:
    """A mixture-of-experts block (Sec. 5.3) runs moe_top_k expert FFNs per token plus the router.
    trainable_blocks (a list): blocks at or after first_trainable that are not in it are frozen in the
    gradient path and run the input gradients only."""
    D, F = dim, mlp_hidden
    fwd_gemm = fwd_attn = bwd_gemm = bwd_attn = 0.0
    for l, (Ta, Tm) in enumerate(zip(tokens_attn, tokens_mlp)):
        ffn = 2 * Tm * D * F
        if l in moe_blocks:
            ffn = moe_top_k * ffn + Tm * D * n_experts
        g = 2.0 * (4 * Ta * D * D + ffn)                 # QKV + proj + fc1 + fc2 (or experts + router)
        a = 4.0 * Ta * Ta * D                            # Q K^T and P V over all heads
        fwd_gemm += g
        fwd_attn += a
        if l >= first_trainable:
            trained = (l in trainable_blocks) if trainable_blocks else True
            bwd_gemm += (2.0 if trained else 1.0) * g    # dgrad + wgrad of every linear (Eq. 2, 4), or dgrad only
            bwd_attn += 2.5 * a                          # dV, dP, dQ, dK and the recomputed Q K^T
    stem = 2.0 * n_patches * patch_dim * D
    head = 3 * 2.0 * D * num_classes
    per_image = dict(fwd_gemm=fwd_gemm + stem, fwd_attn=fwd_attn, bwd_gemm=bwd_gemm, bwd_attn=bwd_attn,
                     head=head)
    out = {k: v * batch for k, v in per_image.items()}
    out["total"] = sum(out.values())
    return out
