"""ctypes binding of include/bsr.h.  Argument marshalling only: tensors are torch CUDA tensors used
as device memory, the stream is torch's current HIP stream.  Same names as the C entry points."""
from __future__ import annotations

import ctypes as C
import os

MAX_BLOCKS = 16
BSR_BF16, BSR_FP32 = 0, 1
BSR_LOSS_CE, BSR_LOSS_MEAN_SQ = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))

BLOCK_FIELDS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj",
                "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")
STEM_FIELDS = ("w_patch", "b_patch", "cls", "pos")
HEAD_FIELDS = ("lnf_g", "lnf_b", "w_head", "b_head")


class BsrError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"bsr error {code}: {text}")
        self.code = code


class bsr_config(C.Structure):
    _fields_ = [("image_size", C.c_int32), ("patch_size", C.c_int32), ("in_chans", C.c_int32),
                ("tokens_in", C.c_int32), ("dim", C.c_int32), ("heads", C.c_int32),
                ("mlp_hidden", C.c_int32), ("depth", C.c_int32), ("num_classes", C.c_int32),
                ("max_batch", C.c_int32), ("n_drop", C.c_int32),
                ("drop_blocks", C.c_int32 * MAX_BLOCKS), ("keep_k", C.c_int32 * MAX_BLOCKS),
                ("keep_ratio", C.c_float), ("first_trainable_block", C.c_int32),
                ("dtype", C.c_int32), ("loss", C.c_int32), ("ln_eps", C.c_float),
                ("n_experts", C.c_int32), ("moe_top_k", C.c_int32), ("n_moe", C.c_int32),
                ("moe_blocks", C.c_int32 * MAX_BLOCKS),
                ("n_trainable", C.c_int32), ("trainable_blocks", C.c_int32 * MAX_BLOCKS),
                ("fuse_dropped", C.c_int32), ("fold_frozen_layernorm", C.c_int32)]


class bsr_tile_choice(C.Structure):
    _fields_ = [("rows", C.c_int32), ("out", C.c_int32), ("in_", C.c_int32), ("tile", C.c_int32),
                ("microseconds", C.c_float)]


class bsr_block_params(C.Structure):
    _fields_ = [(f, C.c_void_p) for f in BLOCK_FIELDS] + [("w_router", C.c_void_p)]


class bsr_params(C.Structure):
    _fields_ = ([(f, C.c_void_p) for f in STEM_FIELDS] + [("blocks", bsr_block_params * MAX_BLOCKS)]
                + [(f, C.c_void_p) for f in HEAD_FIELDS])


def lib_path() -> str:
    return os.path.join(_HERE, "libbsr_hip.so")


_lib = None


def load_library():
    """Load libbsr_hip.so.  Fails loudly when it has not been built (there is no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: run `python -m paper_2405_10951_amd.build` "
                                "(or __graft_entry__.build()) first")
    lib = C.CDLL(path)
    lib.bsr_last_error.restype = C.c_char_p
    lib.bsr_last_error.argtypes = [C.c_void_p]
    for name in ("bsr_token_schedule", "bsr_workspace_bytes", "bsr_init", "bsr_refresh_weights",
                 "bsr_forward_frozen", "bsr_select_tokens", "bsr_train_blocks_fwd_bwd",
                 "bsr_sgd_step", "bsr_destroy", "bsr_profile_begin", "bsr_profile_end", "bsr_moe_routing_io",
                 "bsr_adamw_step", "bsr_saved_activation_bytes", "bsr_autotune", "bsr_autotune_overlapped",
                 "bsr_pipeline_step"):
        getattr(lib, name).restype = C.c_int32
    lib.bsr_token_schedule.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.bsr_workspace_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_size_t)]
    lib.bsr_saved_activation_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    lib.bsr_init.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_void_p)]
    lib.bsr_refresh_weights.argtypes = [C.c_void_p, C.c_void_p]
    lib.bsr_forward_frozen.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p]
    lib.bsr_select_tokens.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                      C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.bsr_train_blocks_fwd_bwd.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.c_void_p]
    lib.bsr_sgd_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_float, C.c_float, C.c_void_p]
    lib.bsr_destroy.argtypes = [C.c_void_p]
    lib.bsr_moe_routing_io.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.bsr_adamw_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_float, C.c_float,
                                   C.c_float, C.c_float, C.c_int32, C.c_void_p]
    lib.bsr_autotune.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.c_void_p, C.c_void_p, C.c_void_p]
    lib.bsr_tile_choices.restype = C.c_int32
    lib.bsr_tile_choices.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32]
    lib.bsr_autotune_overlapped.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.bsr_pipeline_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_float, C.c_float, C.c_float, C.c_void_p, C.c_void_p]
    lib.bsr_linear_forward.restype = C.c_int32
    lib.bsr_linear_forward.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                       C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    lib.bsr_gemm_tile_shapes.restype = C.c_int32
    lib.bsr_gemm_tile_shapes.argtypes = [C.c_void_p, C.c_int32]
    lib.bsr_ln_linear_fold.restype = C.c_int32
    lib.bsr_ln_linear_fold.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p]
    lib.bsr_ln_linear_forward.restype = C.c_int32
    lib.bsr_ln_linear_forward.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_float, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]
    lib.bsr_linear_dgrad.restype = C.c_int32
    lib.bsr_linear_dgrad.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    lib.bsr_linear_wgrad.restype = C.c_int32
    lib.bsr_linear_wgrad.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.bsr_linear_wgrad_static.restype = C.c_int32
    lib.bsr_linear_wgrad_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_void_p]
    lib.bsr_attention_forward.restype = C.c_int32
    lib.bsr_attention_forward.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.bsr_attention_backward.restype = C.c_int32
    lib.bsr_attention_backward.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                           C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.bsr_profile_begin.argtypes = [C.c_void_p]
    lib.bsr_profile_end.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    _lib = lib
    return lib


def make_config(cfg: dict, max_batch: int, keep_k=None) -> bsr_config:
    """Fill a bsr_config from a plain dict (the keys of the C struct; `first_trainable` is accepted
    for first_trainable_block, dtype may be "bf16"/"fp32")."""
    c = bsr_config()
    for f in ("image_size", "patch_size", "in_chans", "tokens_in", "dim", "heads", "mlp_hidden",
              "depth", "num_classes", "loss"):
        setattr(c, f, int(cfg.get(f, 0)))
    c.max_batch = int(max_batch)
    c.first_trainable_block = int(cfg.get("first_trainable_block", cfg.get("first_trainable", 0)))
    dt = cfg.get("dtype", "bf16")
    c.dtype = {"bf16": BSR_BF16, "fp32": BSR_FP32}.get(dt, dt)
    c.keep_ratio = float(cfg.get("keep_ratio", 1.0))
    c.ln_eps = float(cfg.get("ln_eps", 1e-6))
    drops = list(cfg.get("drop_blocks", []))
    c.n_drop = len(drops)
    for i, b in enumerate(drops):
        c.drop_blocks[i] = int(b)
    if keep_k is None:
        keep_k = cfg.get("keep_k")
    if keep_k:
        for i, k in enumerate(keep_k):
            c.keep_k[i] = int(k)
    moe = list(cfg.get("moe_blocks", []))
    c.n_moe = len(moe)
    for i, b in enumerate(moe):
        c.moe_blocks[i] = int(b)
    c.n_experts = int(cfg.get("n_experts", 0))
    c.moe_top_k = int(cfg.get("moe_top_k", 0))
    c.fuse_dropped = int(bool(cfg.get("fuse_dropped", 0)))
    c.fold_frozen_layernorm = int(bool(cfg.get("fold_frozen_layernorm", 0)))
    tb = list(cfg.get("trainable_blocks") or [])
    c.n_trainable = len(tb)
    for i, b in enumerate(tb):
        c.trainable_blocks[i] = int(b)
    if tb:
        c.first_trainable_block = int(tb[0])
    return c


def _check(rc, ctx=None):
    if rc != 0:
        raise BsrError(rc, load_library().bsr_last_error(ctx).decode())


def bsr_token_schedule(cfg: bsr_config):
    """-> (keep_k per drop, tokens seen by MHSA per block, tokens seen by the FFN per block)."""
    lib = load_library()
    kk = (C.c_int32 * MAX_BLOCKS)()
    ta = (C.c_int32 * MAX_BLOCKS)()
    tm = (C.c_int32 * MAX_BLOCKS)()
    _check(lib.bsr_token_schedule(C.byref(cfg), kk, ta, tm))
    return list(kk[:cfg.n_drop]), list(ta[:cfg.depth]), list(tm[:cfg.depth])


def bsr_workspace_bytes(cfg: bsr_config) -> int:
    n = C.c_size_t(0)
    _check(load_library().bsr_workspace_bytes(C.byref(cfg), C.byref(n)))
    return int(n.value)


class bsr_saved_bytes(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("qkv", "softmax", "attn_out", "gelu_in", "linear_in", "residual",
                                          "stats", "moe", "total")]


def bsr_saved_activation_bytes(cfg: bsr_config, batch: int):
    """-> (list per block of dict kind -> bytes, dict of sums) for `batch` images."""
    per = (bsr_saved_bytes * MAX_BLOCKS)()
    tot = bsr_saved_bytes()
    _check(load_library().bsr_saved_activation_bytes(C.byref(cfg), C.c_int32(batch), per, C.byref(tot)))
    as_dict = lambda r: {n: int(getattr(r, n)) for n, _ in bsr_saved_bytes._fields_}
    return [as_dict(per[l]) for l in range(cfg.depth)], as_dict(tot)


def _cur_stream(t):
    import torch
    return C.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def bsr_linear_forward(x, w_t, bias=None, act=0, u_out=None, res=None, y=None, tile=0):
    """x [M,in] bf16, w_t [out,in] bf16 -> (y [M,out] bf16, used_mfma).  tile: 0 or a block-tile shape id."""
    import torch
    M, kin = x.shape
    out = w_t.shape[0]
    if y is None:
        y = torch.empty((M, out), dtype=torch.bfloat16, device=x.device)
    used = C.c_int32(-1)
    _check(load_library().bsr_linear_forward(_dp(x), M, kin, out, _dp(w_t), _dp(bias), act, _dp(u_out),
                                             _dp(res), _dp(y), tile, C.byref(used), _cur_stream(x)))
    return y, used.value


def bsr_gemm_tile_shapes():
    """Ids of the block-tile shapes of the bf16 product kernel."""
    lib = load_library()
    n = lib.bsr_gemm_tile_shapes(None, 0)
    ids = (C.c_int32 * n)()
    lib.bsr_gemm_tile_shapes(ids, n)
    return list(ids)


def bsr_ln_linear_fold(w, bias, gamma, beta):
    """w [in,out], bias [out], gamma [in], beta [in] fp32 -> (w_folded [out,in] bf16, colsum [out], bias_folded [out])."""
    import torch
    kin, out = w.shape
    wf = torch.empty((out, kin), dtype=torch.bfloat16, device=w.device)
    cs = torch.empty(out, dtype=torch.float32, device=w.device)
    bf = torch.empty(out, dtype=torch.float32, device=w.device)
    _check(load_library().bsr_ln_linear_fold(_dp(w), _dp(bias), _dp(gamma), _dp(beta), kin, out, _dp(wf), _dp(cs),
                                             _dp(bf), _cur_stream(w)))
    return wf, cs, bf


def bsr_ln_linear_forward(x, w_folded, colsum, bias_folded, eps=1e-6, act=0, tile=0, y=None):
    """x [M,in] bf16 and the folded tensors -> y [M,out] bf16 = act(LN(x) W + b)."""
    import torch
    M, kin = x.shape
    out = w_folded.shape[0]
    if y is None:
        y = torch.empty((M, out), dtype=torch.bfloat16, device=x.device)
    _check(load_library().bsr_ln_linear_forward(_dp(x), M, kin, out, _dp(w_folded), _dp(colsum), _dp(bias_folded),
                                                C.c_float(eps), act, _dp(y), tile, _cur_stream(x)))
    return y


def bsr_linear_dgrad(dy, w_s, u=None, dx=None, tile=0):
    """dy [M,out] bf16, w_s [in,out] bf16 -> (dx [M,in] bf16, used_mfma).  tile: 0 or a block-tile shape id."""
    import torch
    M, out = dy.shape
    kin = w_s.shape[0]
    if dx is None:
        dx = torch.empty((M, kin), dtype=torch.bfloat16, device=dy.device)
    used = C.c_int32(-1)
    _check(load_library().bsr_linear_dgrad(_dp(dy), M, kin, out, _dp(w_s), _dp(u), _dp(dx), tile, C.byref(used),
                                           _cur_stream(dy)))
    return dx, used.value


def bsr_linear_wgrad(x, dy, dw=None, workspace=None, db=None):
    """x [M,in], dy [M,out] bf16 -> (dw [in,out] fp32, used_mfma).  workspace: fp32 tensor or None;
    db: fp32 [out] tensor that receives the bias gradient, or None."""
    import torch
    M, kin = x.shape
    out = dy.shape[1]
    if dw is None:
        dw = torch.empty((kin, out), dtype=torch.float32, device=x.device)
    used = C.c_int32(-1)
    _check(load_library().bsr_linear_wgrad(_dp(x), _dp(dy), M, kin, out, _dp(dw), _dp(db), _dp(workspace),
                                           C.c_size_t(0 if workspace is None else workspace.numel()),
                                           C.byref(used), _cur_stream(x)))
    return dw, used.value


def bsr_linear_wgrad_static(x, dy, dw=None, db=None):
    """bsr_linear_wgrad with the split-K partial sums in the library's built-in scratch array: the call itself
    allocates nothing (dw and db, when not given, are allocated here, in the binding)."""
    import torch
    M, kin = x.shape
    out = dy.shape[1]
    if dw is None:
        dw = torch.empty((kin, out), dtype=torch.float32, device=x.device)
    used = C.c_int32(-1)
    _check(load_library().bsr_linear_wgrad_static(_dp(x), _dp(dy), M, kin, out, _dp(dw), _dp(db), C.byref(used),
                                                  _cur_stream(x)))
    return dw, used.value


def bsr_attention_forward(qkv, heads, want_lse=True, want_cls=True):
    """qkv [B,T,3D] bf16 -> (out [B,T,D] bf16, lse [B,H,T] | None, cls_prob [B,H,T] | None, used_mfma)."""
    import torch
    B, T, D3 = qkv.shape
    D = D3 // 3
    out = torch.empty((B, T, D), dtype=torch.bfloat16, device=qkv.device)
    lse = torch.empty((B, heads, T), dtype=torch.float32, device=qkv.device) if want_lse else None
    cls = torch.empty((B, heads, T), dtype=torch.float32, device=qkv.device) if want_cls else None
    used = C.c_int32(-1)
    _check(load_library().bsr_attention_forward(_dp(qkv), B, T, heads, D // heads, _dp(out), _dp(lse), _dp(cls),
                                                C.byref(used), _cur_stream(qkv)))
    return out, lse, cls, used.value


def bsr_attention_backward(qkv, out, dout, lse, heads):
    """-> (dqkv [B,T,3D] bf16, used_mfma)."""
    import torch
    B, T, D3 = qkv.shape
    D = D3 // 3
    dqkv = torch.empty_like(qkv)
    delta = torch.empty((B, heads, T), dtype=torch.float32, device=qkv.device)
    used = C.c_int32(-1)
    _check(load_library().bsr_attention_backward(_dp(qkv), _dp(out), _dp(dout), _dp(lse), B, T, heads, D // heads,
                                                 _dp(delta), _dp(dqkv), C.byref(used), _cur_stream(qkv)))
    return dqkv, used.value


def _params_struct(tensors: dict) -> bsr_params:
    p = bsr_params()
    for name, t in tensors.items():
        if t is None:
            continue
        ptr = t.data_ptr()
        if name.startswith("blocks."):
            _, i, leaf = name.split(".")
            setattr(p.blocks[int(i)], leaf, ptr)
        else:
            setattr(p, name, ptr)
    return p


def _dp(t):
    return None if t is None else C.c_void_p(t.data_ptr())


class Context:
    """Owns a bsr_ctx and the torch tensors (device memory) it points into.  Methods carry the
    names of the C entry points and forward to them one to one."""

    def __init__(self, cfg: dict, params: dict, max_batch: int, keep_k=None, device="cuda:0"):
        import torch
        self.torch = torch
        self.lib = load_library()
        self.device = torch.device(device)
        self.c = make_config(cfg, max_batch, keep_k)
        self.act_dtype = torch.float32 if self.c.dtype == BSR_FP32 else torch.bfloat16
        self.keep_k, self.tokens_attn, self.tokens_mlp = bsr_token_schedule(self.c)
        # master weights: fp32 device tensors owned here, updated in place by bsr_sgd_step
        self.params = {k: torch.as_tensor(v, dtype=torch.float32).to(self.device).contiguous()
                       for k, v in params.items()}
        self._pstruct = _params_struct(self.params)
        nbytes = bsr_workspace_bytes(self.c)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = (self.workspace.data_ptr() + 255) & ~255
        self.ctx = C.c_void_p()
        _check(self.lib.bsr_init(C.byref(self.c), C.byref(self._pstruct), C.c_void_p(base),
                                 C.c_size_t(nbytes), self._stream(), C.byref(self.ctx)))
        ft, L = self.c.first_trainable_block, self.c.depth
        self.T_f = self.tokens_attn[ft] if ft < L else self.tokens_mlp[L - 1]
        self.T_last = self.tokens_mlp[L - 1]
        self.frozen_drops = [i for i in range(self.c.n_drop) if self.c.drop_blocks[i] < ft]
        self.train_drops = [i for i in range(self.c.n_drop) if self.c.drop_blocks[i] >= ft]
        tb = [self.c.trainable_blocks[i] for i in range(self.c.n_trainable)]
        self.trainable_names = [n for n in self.params if n in HEAD_FIELDS or
                                (n.startswith("blocks.") and
                                 ((int(n.split(".")[1]) in tb) if tb else int(n.split(".")[1]) >= ft))]

    def _stream(self):
        return C.c_void_p(self.torch.cuda.current_stream(self.device).cuda_stream)

    def _chk(self, rc):
        _check(rc, self.ctx)

    def n_in(self, drop_i: int) -> int:
        """patch tokens entering drop location drop_i"""
        return self.tokens_attn[self.c.drop_blocks[drop_i]] - 1

    def new_grads(self) -> dict:
        return {n: self.torch.zeros_like(self.params[n]) for n in self.trainable_names}

    def moe_rows(self, B: int) -> dict:
        """block -> number of token rows (B * tokens of its FFN) for every mixture-of-experts block"""
        return {self.c.moe_blocks[i]: B * self.tokens_mlp[self.c.moe_blocks[i]] for i in range(self.c.n_moe)}

    # ---- entry points ---------------------------------------------------------------------
    def bsr_moe_routing_io(self, forced_experts=None, experts_out=None, router_logits_out=None):
        """Device tensors laid out block after block over the mixture-of-experts blocks (see bsr.h);
        the context only keeps the pointers, so the tensors are kept alive here."""
        self._moe_io = (forced_experts, experts_out, router_logits_out)
        self._chk(self.lib.bsr_moe_routing_io(self.ctx, _dp(forced_experts), _dp(experts_out),
                                              _dp(router_logits_out)))

    def bsr_refresh_weights(self):
        self._chk(self.lib.bsr_refresh_weights(self.ctx, self._stream()))

    def bsr_forward_frozen(self, inp, x_out=None, kept_idx_out=None, scores_out=None, forced_idx=None):
        t = self.torch
        B = inp.shape[0]
        if x_out is None:
            x_out = t.empty((B, self.T_f, self.c.dim), dtype=self.act_dtype, device=self.device)
        self._chk(self.lib.bsr_forward_frozen(self.ctx, _dp(inp), B, _dp(x_out), _dp(kept_idx_out),
                                              _dp(scores_out), _dp(forced_idx), self._stream()))
        return x_out

    def bsr_select_tokens(self, cls_attn, x_in, k, idx_out=None, x_out=None):
        t = self.torch
        B, n = cls_attn.shape
        if idx_out is None:
            idx_out = t.empty((B, max(k, 1)), dtype=t.int32, device=self.device)
        if x_in is not None and x_out is None:
            x_out = t.empty((B, k + 1, self.c.dim), dtype=self.act_dtype, device=self.device)
        self._chk(self.lib.bsr_select_tokens(self.ctx, _dp(cls_attn), _dp(x_in), B, n, k, _dp(idx_out),
                                             _dp(x_out), self._stream()))
        return idx_out[:, :k], x_out

    def bsr_train_blocks_fwd_bwd(self, x_in, labels, grads: dict, loss_out=None, logits_out=None,
                                 x_final_out=None, kept_idx_out=None, scores_out=None, forced_idx=None):
        t = self.torch
        B = x_in.shape[0]
        if loss_out is None:
            loss_out = t.zeros(4, dtype=t.float32, device=self.device)
        gs = _params_struct(grads)
        self._chk(self.lib.bsr_train_blocks_fwd_bwd(self.ctx, _dp(x_in), _dp(labels), B, _dp(loss_out),
                                                    _dp(logits_out), _dp(x_final_out), C.byref(gs),
                                                    _dp(kept_idx_out), _dp(scores_out), _dp(forced_idx),
                                                    self._stream()))
        return loss_out

    def bsr_sgd_step(self, grads: dict, momenta: dict | None, lr: float, momentum: float = 0.0,
                     weight_decay: float = 0.0):
        gs = _params_struct(grads)
        ms = _params_struct(momenta) if momenta is not None else None
        self._chk(self.lib.bsr_sgd_step(self.ctx, C.byref(gs), C.byref(ms) if ms is not None else None,
                                        C.c_float(lr), C.c_float(momentum), C.c_float(weight_decay),
                                        self._stream()))

    def bsr_autotune(self, inp, labels, x_frozen, loss_out, grads: dict):
        """-> (launches with a measured tile choice, how many differ from the cost model's)."""
        gs = _params_struct(grads)
        n, ch = C.c_int32(0), C.c_int32(0)
        self._chk(self.lib.bsr_autotune(self.ctx, _dp(inp), _dp(labels), C.c_int32(inp.shape[0]), _dp(x_frozen),
                                        _dp(loss_out), C.byref(gs), C.byref(n), C.byref(ch), self._stream()))
        return int(n.value), int(ch.value)

    def bsr_tile_choices(self, part: int):
        """[(rows, out, in, tile, microseconds)] of the launches of part 0 (frozen prefix) or 1 (trainable part)."""
        n = self.lib.bsr_tile_choices(self.ctx, part, None, 0)
        buf = (bsr_tile_choice * max(n, 1))()
        self.lib.bsr_tile_choices(self.ctx, part, buf, n)
        return [(b.rows, b.out, b.in_, b.tile, b.microseconds) for b in buf[:n]]

    def bsr_pipeline_step(self, inp_next, x_next, x_cur, labels_cur, loss_out, grads: dict, momenta: dict | None, lr: float,
                          momentum: float, weight_decay: float, stream_frozen, stream_train):
        """Frozen prefix of the next batch (inp_next -> x_next, both None on the last step) on stream_frozen beside
        the trainable part + SGD step of the current batch (x_cur, None on the first call) on stream_train
        (two torch streams)."""
        gs = _params_struct(grads)
        ms = _params_struct(momenta) if momenta is not None else None
        B = (inp_next if inp_next is not None else x_cur).shape[0]
        self._chk(self.lib.bsr_pipeline_step(self.ctx, _dp(inp_next), _dp(x_next), _dp(x_cur), _dp(labels_cur), C.c_int32(B),
                                             _dp(loss_out), C.byref(gs), C.byref(ms) if ms is not None else None,
                                             C.c_float(lr), C.c_float(momentum), C.c_float(weight_decay),
                                             C.c_void_p(stream_frozen.cuda_stream), C.c_void_p(stream_train.cuda_stream)))

    def bsr_autotune_overlapped(self, inp, labels, x_frozen, x_side, loss_out, grads: dict, side_stream):
        """Tile choice timed with the frozen prefix (current stream) beside the trainable part (side_stream, a
        torch stream); -> (launches with a measured tile choice, how many differ from the cost model's)."""
        gs = _params_struct(grads)
        n, ch = C.c_int32(0), C.c_int32(0)
        self._chk(self.lib.bsr_autotune_overlapped(self.ctx, _dp(inp), _dp(labels), C.c_int32(inp.shape[0]), _dp(x_frozen),
                                                   _dp(x_side), _dp(loss_out), C.byref(gs), C.byref(n), C.byref(ch),
                                                   self._stream(), C.c_void_p(side_stream.cuda_stream)))
        return int(n.value), int(ch.value)

    def bsr_adamw_step(self, grads: dict, exp_avg: dict, exp_avg_sq: dict, lr: float, beta1: float = 0.9,
                       beta2: float = 0.999, eps: float = 1e-8, weight_decay: float = 0.01, step: int = 1):
        gs, ms, vs = _params_struct(grads), _params_struct(exp_avg), _params_struct(exp_avg_sq)
        self._chk(self.lib.bsr_adamw_step(self.ctx, C.byref(gs), C.byref(ms), C.byref(vs), C.c_float(lr),
                                          C.c_float(beta1), C.c_float(beta2), C.c_float(eps),
                                          C.c_float(weight_decay), C.c_int32(step), self._stream()))

    def bsr_profile_begin(self):
        self._chk(self.lib.bsr_profile_begin(self.ctx))

    def bsr_profile_end(self) -> dict:
        """-> {class: (ms, flops, launches)} for gemm / attn_fwd / attn_bwd; waits for the stream."""
        ms = (C.c_double * 3)()
        fl = (C.c_double * 3)()
        n = (C.c_int32 * 3)()
        self._chk(self.lib.bsr_profile_end(self.ctx, ms, fl, n))
        return {name: (ms[i], fl[i], n[i]) for i, name in enumerate(("gemm", "attn_fwd", "attn_bwd"))}

    def bsr_destroy(self):
        if self.ctx:
            self.lib.bsr_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.bsr_destroy()
        except Exception:
            pass
