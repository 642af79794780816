"""Seeded synthetic inputs for the BSR fine-tuning step (shapes of Sec. 5's ViT-B / DeiT-S runs).

This module only draws random numbers and names tensors.  It holds none of the
method's arithmetic (no token schedule, no attention, no selection): the CPU
oracle and the HIP library each derive those on their own.  Both sides receive
the same numpy arrays from here, so a disagreement between them can never come
from the inputs.

Parameter tensors (all float32, linears row-major [in, out]):
  stem   : w_patch [C*P*P, D]  b_patch [D]  cls [D]  pos [T, D]
  block i: ln1_g ln1_b [D]  w_qkv [D, 3D]  b_qkv [3D]  w_proj [D, D]  b_proj [D]
           ln2_g ln2_b [D]  w_fc1 [D, F]   b_fc1 [F]   w_fc2 [F, D]   b_fc2 [D]
  head   : lnf_g lnf_b [D]  w_head [D, C]  b_head [C]
Columns of w_qkv are ordered [q | k | v], each split into H heads of d = D/H.
A mixture-of-experts block (config keys n_experts, moe_top_k, moe_blocks) holds one FFN per expert
and a router: w_router [D, E]  w_fc1 [E, D, F]  b_fc1 [E, F]  w_fc2 [E, F, D]  b_fc2 [E, D].
"""
from __future__ import annotations

import copy
import numpy as np

BLOCK_TENSORS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj",
                 "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")
MOE_TENSORS = ("w_router",)      # present in mixture-of-experts blocks only
STEM_TENSORS = ("w_patch", "b_patch", "cls", "pos")
HEAD_TENSORS = ("lnf_g", "lnf_b", "w_head", "b_head")

LOSS_CE = 0
LOSS_MEAN_SQ = 1

# The workloads.  drop_blocks / first_trainable are 0-based block indices.
CONFIGS = {
    # one encoder block on token input, fp32, drop inside the (trainable) block
    "c1_block_fp32": dict(image_size=0, patch_size=0, in_chans=0, tokens_in=65,
                          dim=192, heads=3, mlp_hidden=768, depth=1, num_classes=0,
                          drop_blocks=[0], keep_ratio=0.7, first_trainable=0,
                          dtype="fp32", loss=LOSS_MEAN_SQ, batch=2),
    # DeiT-S shape
    "c2_deit_s": dict(image_size=224, patch_size=16, in_chans=3, tokens_in=0,
                      dim=384, heads=6, mlp_hidden=1536, depth=12, num_classes=10,
                      drop_blocks=[3, 6, 9], keep_ratio=0.7, first_trainable=8,
                      dtype="bf16", loss=LOSS_CE, batch=32),
    # ViT-B/16 shape: the headline workload
    "c3_vit_b": dict(image_size=224, patch_size=16, in_chans=3, tokens_in=0,
                     dim=768, heads=12, mlp_hidden=3072, depth=12, num_classes=100,
                     drop_blocks=[3, 6, 9], keep_ratio=0.7, first_trainable=8,
                     dtype="bf16", loss=LOSS_CE, batch=32),
    # small multi-block models for quick parity and gradient checks
    "tiny_2blk": dict(image_size=16, patch_size=4, in_chans=3, tokens_in=0,
                      dim=32, heads=2, mlp_hidden=64, depth=2, num_classes=5,
                      drop_blocks=[1], keep_ratio=0.6, first_trainable=0,
                      dtype="fp32", loss=LOSS_CE, batch=3),
    "mini_4blk": dict(image_size=64, patch_size=8, in_chans=3, tokens_in=0,
                      dim=128, heads=4, mlp_hidden=256, depth=4, num_classes=10,
                      drop_blocks=[1, 2], keep_ratio=0.7, first_trainable=2,
                      dtype="fp32", loss=LOSS_CE, batch=5),
    # ViT-S shape with a 16-expert, top-2 mixture-of-experts FFN in every other block (Sec. 5.3 shape
    # of the method; expert count from the paper, top-2 softmax gating as the workload states it)
    "c5_vit_s_moe": dict(image_size=224, patch_size=16, in_chans=3, tokens_in=0,
                         dim=384, heads=6, mlp_hidden=1536, depth=12, num_classes=100,
                         drop_blocks=[3, 6, 9], keep_ratio=0.7, first_trainable=8,
                         n_experts=16, moe_top_k=2, moe_blocks=[1, 3, 5, 7, 9, 11],
                         dtype="bf16", loss=LOSS_CE, batch=32),
    # the paper's default layout (Sec. 5, Table 7): every fourth block trained, the blocks between
    # them frozen but in the gradient path (input gradients only, Eq. 2 / Eq. 3), drop rate 0.5
    "c6_vit_b_interleaved": dict(image_size=224, patch_size=16, in_chans=3, tokens_in=0,
                                 dim=768, heads=12, mlp_hidden=3072, depth=12, num_classes=100,
                                 drop_blocks=[3, 6, 9], keep_ratio=0.5, first_trainable=3,
                                 trainable_blocks=[3, 7, 11], dtype="bf16", loss=LOSS_CE, batch=32),
    "mini_interleaved": dict(image_size=64, patch_size=8, in_chans=3, tokens_in=0,
                             dim=128, heads=2, mlp_hidden=256, depth=6, num_classes=10,
                             drop_blocks=[1, 3], keep_ratio=0.6, first_trainable=1,
                             trainable_blocks=[1, 3, 5], dtype="fp32", loss=LOSS_CE, batch=5),
    # small mixture-of-experts models
    "tiny_moe": dict(image_size=16, patch_size=4, in_chans=3, tokens_in=0,
                     dim=32, heads=2, mlp_hidden=48, depth=3, num_classes=5,
                     drop_blocks=[1], keep_ratio=0.6, first_trainable=0,
                     n_experts=4, moe_top_k=2, moe_blocks=[0, 2],
                     dtype="fp32", loss=LOSS_CE, batch=3),
    "mini_moe": dict(image_size=64, patch_size=8, in_chans=3, tokens_in=0,
                     dim=128, heads=2, mlp_hidden=256, depth=4, num_classes=10,
                     drop_blocks=[1, 2], keep_ratio=0.7, first_trainable=2,
                     n_experts=8, moe_top_k=2, moe_blocks=[1, 3],
                     dtype="bf16", loss=LOSS_CE, batch=6),
}


def get_config(name: str, **overrides) -> dict:
    cfg = copy.deepcopy(CONFIGS[name])
    cfg.update(overrides)
    cfg["name"] = name
    return cfg


def is_trainable_block(cfg: dict, l: int) -> bool:
    """Blocks listed in trainable_blocks, or (no list) every block from first_trainable on."""
    tb = cfg.get("trainable_blocks")
    return (l in tb) if tb else (l >= cfg["first_trainable"])


def tokens_at_input(cfg: dict) -> int:
    """T = N + 1 tokens entering block 0 (Sec. 3.1)."""
    if cfg["image_size"] == 0:
        return cfg["tokens_in"]
    g = cfg["image_size"] // cfg["patch_size"]
    return g * g + 1


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16-representable value (ties to even), kept as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    bias = ((u >> 16) & 1) + 0x7FFF
    r = ((u + bias) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(a.shape)


def param_shapes(cfg: dict) -> dict:
    D, F, C = cfg["dim"], cfg["mlp_hidden"], cfg["num_classes"]
    shapes = {}
    if cfg["image_size"]:
        pdim = cfg["in_chans"] * cfg["patch_size"] ** 2
        shapes.update({"w_patch": (pdim, D), "b_patch": (D,), "cls": (D,),
                       "pos": (tokens_at_input(cfg), D)})
    E = cfg.get("n_experts", 0)
    for i in range(cfg["depth"]):
        pre = f"blocks.{i}."
        shapes.update({pre + "ln1_g": (D,), pre + "ln1_b": (D,),
                       pre + "w_qkv": (D, 3 * D), pre + "b_qkv": (3 * D,),
                       pre + "w_proj": (D, D), pre + "b_proj": (D,),
                       pre + "ln2_g": (D,), pre + "ln2_b": (D,)})
        if E and i in cfg.get("moe_blocks", ()):
            shapes.update({pre + "w_router": (D, E),
                           pre + "w_fc1": (E, D, F), pre + "b_fc1": (E, F),
                           pre + "w_fc2": (E, F, D), pre + "b_fc2": (E, D)})
        else:
            shapes.update({pre + "w_fc1": (D, F), pre + "b_fc1": (F,),
                           pre + "w_fc2": (F, D), pre + "b_fc2": (D,)})
    if C:
        shapes.update({"lnf_g": (D,), "lnf_b": (D,), "w_head": (D, C), "b_head": (C,)})
    return shapes


def make_params(cfg: dict, seed: int = 0, std: float = 0.02, peaky: float = 1.0,
                bf16_exact: bool | None = None) -> dict:
    """Draw every parameter tensor ~ N(0, std^2) (LayerNorm gains 1 + N(0, std^2)), in the fixed
    order of param_shapes().  peaky > 1 scales the q and k columns of every w_qkv so that attention
    logits spread the way a trained model's do.  bf16_exact rounds each value once to bf16."""
    if bf16_exact is None:
        bf16_exact = cfg["dtype"] == "bf16"
    rng = np.random.default_rng(seed)
    out = {}
    D = cfg["dim"]
    for name, shape in param_shapes(cfg).items():
        a = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        leaf = name.split(".")[-1]
        if leaf in ("ln1_g", "ln2_g", "lnf_g"):
            a = a + np.float32(1.0)
        if leaf == "w_qkv" and peaky != 1.0:
            a[:, : 2 * D] *= np.float32(peaky)
        if leaf == "w_router":   # N(0, 1/D): router logits of a normalised token are ~ N(0, 1)
            a = a * np.float32(1.0 / (std * np.sqrt(D)))
        out[name] = round_to_bf16(a) if bf16_exact else a
    return out


def make_inputs(cfg: dict, batch: int | None = None, seed: int = 0,
                bf16_exact: bool | None = None):
    """Images [B, C, H, W] ~ N(0,1) (or tokens [B, T, D] ~ N(0,1) when the config has no stem) and
    labels uniform in [0, num_classes)."""
    if bf16_exact is None:
        bf16_exact = cfg["dtype"] == "bf16"
    B = cfg["batch"] if batch is None else batch
    rng = np.random.default_rng(seed + 1_000_003)
    if cfg["image_size"]:
        x = rng.standard_normal((B, cfg["in_chans"], cfg["image_size"], cfg["image_size"]),
                                dtype=np.float32)
    else:
        x = rng.standard_normal((B, cfg["tokens_in"], cfg["dim"]), dtype=np.float32)
    if bf16_exact:
        x = round_to_bf16(x)
    C = max(cfg["num_classes"], 1)
    labels = rng.integers(0, C, size=(B,), dtype=np.int64).astype(np.int32)
    return x, labels
