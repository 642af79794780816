"""Closed-form bookkeeping of the BSR step, used only to pin the oracle's reading of the paper
against the numbers the paper prints (Table 1, the GMACs columns of Tables 3, 4 and 8).
TEST INFRASTRUCTURE ONLY."""
from __future__ import annotations


def tokens_per_block(T0: int, depth: int, drop_blocks, keep_k):
    """(T seen by MHSA, T seen by the FFN) for every block; a drop location shrinks T between its
    MHSA and its FFN (Sec. 4.3, Discussion 3)."""
    out, T, di = [], T0, 0
    drops = list(drop_blocks)
    for l in range(depth):
        Ta = T
        if di < len(drops) and drops[di] == l:
            T = keep_k[di] + 1
            di += 1
        out.append((Ta, T))
    return out


def forward_macs(T_blocks, D: int, F: int, n_patches: int, patch_dim: int, num_classes: int) -> int:
    """Multiply-accumulates of one image's forward pass: QKV + proj + FFN linears, Q K^T and P V,
    patch embedding and classifier."""
    macs = n_patches * patch_dim * D + D * num_classes
    for Ta, Tm in T_blocks:
        macs += Ta * 4 * D * D + 2 * Ta * Ta * D + 2 * Tm * D * F
    return macs


def saved_bytes_nonlinear(T: int, D: int, H: int, F: int, bytes_per: int = 4) -> dict:
    """Table 1: what the non-linear layers of one block keep for backward, per image."""
    return {"qkv": 3 * T * D * bytes_per, "softmax_in": H * T * T * bytes_per,
            "gelu_in": T * F * bytes_per}


def saved_bytes_trainable(T: int, D: int, H: int, F: int, bytes_per: int = 4) -> int:
    """A trainable block also keeps the inputs of its linear layers and LayerNorms (Sec. 3.2):
    LN1, QKV, proj, LN2, fc1 inputs [T,D] and the fc2 input [T,F]."""
    nl = saved_bytes_nonlinear(T, D, H, F, bytes_per)
    return sum(nl.values()) + 5 * T * D * bytes_per + T * F * bytes_per


def saved_bytes_lse_design(Ta: int, Tm: int, D: int, H: int, F: int, bytes_per: int, trained: bool,
                           drop: bool, fused: bool = False) -> dict:
    """What a block in the gradient path must keep when the attention backward recomputes the
    probabilities from one log-sum-exp per row instead of storing the [H,T,T] softmax input of
    Table 1.  Ta tokens enter the MHSA, Tm the FFN (Sec. 4.3 Discussion 3).  The non-linear layers
    need Q,K,V, the row statistics, O (for rowsum(dO*O)) and the GELU input; LayerNorm backward
    needs its input (x after MHSA, the block output for the next block's LN1) and mean/rstd; a block
    whose weights are trained also needs the inputs of its four linears (Eq. 4): LN1 output, O
    (already kept), LN2 output, GELU output."""
    e = bytes_per
    out = {"qkv": 3 * Ta * D * e, "softmax": H * Ta * 4, "attn_out": Ta * D * e, "gelu_in": Tm * F * e,
           "linear_in": (Ta * D * e + Tm * D * e + Tm * F * e) if trained else 0,
           "residual": 2 * Tm * D * e,
           "stats": 2 * Ta * 4 + 2 * Tm * 4 + (Tm * 4 if drop else 0) + (Ta * 4 if fused else 0)}
    out["total"] = sum(out.values())
    return out
