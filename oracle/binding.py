"""ctypes access to the C oracle (oracle/bsr_oracle.c).  TEST INFRASTRUCTURE ONLY.

The C file is compiled twice, once with REAL=double and once with REAL=float.  Nothing here does
arithmetic of the method except token_schedule(), the K-from-keep-ratio rule of Sec. 4.1 / 4.3.
"""
from __future__ import annotations

import ctypes as C
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bsr_oracle.c")
MAX_BLOCKS = 16

BLOCK_FIELDS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj",
                "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


def token_schedule(n0: int, keep_ratio: float, n_drop: int, fuse: bool = False) -> list[int]:
    """Patch tokens kept after each drop location: K = floor(r * n) on the current patch count
    (Sec. 4.3, Discussion 3: N/2, N/4, N/8 at drop rate 0.5).  The 1e-9 guards products such as
    0.29 * 100 that land a hair below an integer in binary floating point.  With fuse, the dropped
    tokens of a location become one more patch token of the following blocks."""
    ks, n = [], n0
    for _ in range(n_drop):
        k = int(math.floor(float(keep_ratio) * n + 1e-9))
        ks.append(k)
        n = k + (1 if fuse and n - k > 0 else 0)
    return ks


def _lib_path(prec: str) -> str:
    return os.path.join(_HERE, f"libbsr_oracle_{prec}.so")


def build_oracle(force: bool = False) -> None:
    """gcc -O3 -fopenmp, once per precision."""
    for prec, real in (("f64", "double"), ("f32", "float")):
        out = _lib_path(prec)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               f"-DREAL={real}", "-o", out, _SRC, "-lm"]
        subprocess.run(cmd, check=True)


def build_oracle_sanitized(out_dir: str) -> None:
    """Both precisions with gcc's AddressSanitizer and UndefinedBehaviorSanitizer, into out_dir (load them with
    gcc's libasan and libubsan preloaded)."""
    os.makedirs(out_dir, exist_ok=True)
    for prec, real in (("f64", "double"), ("f32", "float")):
        cmd = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-march=x86-64-v3",
               "-fopenmp", "-fPIC", "-shared", "-std=c11", f"-DREAL={real}", "-o",
               os.path.join(out_dir, f"libbsr_oracle_{prec}.so"), _SRC, "-lm"]
        subprocess.run(cmd, check=True)


class _Config(C.Structure):
    _fields_ = [("image_size", C.c_int32), ("patch_size", C.c_int32), ("in_chans", C.c_int32),
                ("tokens_in", C.c_int32), ("dim", C.c_int32), ("heads", C.c_int32),
                ("mlp_hidden", C.c_int32), ("depth", C.c_int32), ("num_classes", C.c_int32),
                ("n_drop", C.c_int32), ("drop_blocks", C.c_int32 * MAX_BLOCKS),
                ("keep_k", C.c_int32 * MAX_BLOCKS), ("first_trainable", C.c_int32),
                ("loss", C.c_int32), ("ln_eps", C.c_double),
                ("n_experts", C.c_int32), ("moe_top_k", C.c_int32), ("moe_block", C.c_int32 * MAX_BLOCKS),
                ("fuse_dropped", C.c_int32)]


class _Block(C.Structure):
    _fields_ = [(f, C.c_void_p) for f in BLOCK_FIELDS] + [("w_router", C.c_void_p)]


class _Params(C.Structure):
    _fields_ = ([(f, C.c_void_p) for f in ("w_patch", "b_patch", "cls", "pos")]
                + [("blocks", _Block * MAX_BLOCKS)]
                + [(f, C.c_void_p) for f in ("lnf_g", "lnf_b", "w_head", "b_head")])


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Oracle:
    """One precision of the oracle.  All arrays are numpy, C-contiguous, of self.dtype."""

    def __init__(self, precision: str = "f64"):
        assert precision in ("f64", "f32")
        build_oracle()
        self.dtype = np.float64 if precision == "f64" else np.float32
        self.lib = C.CDLL(_lib_path(precision))
        assert self.lib.orc_sizeof_real() == np.dtype(self.dtype).itemsize
        self.lib.orc_step.restype = C.c_int32
        self.lib.orc_step_moe.restype = C.c_int32
        self.lib.orc_cross_entropy.restype = C.c_double if precision == "f64" else C.c_float

    # ---- marshalling -------------------------------------------------------------------
    def arr(self, a):
        return np.ascontiguousarray(a, dtype=self.dtype)

    def _config(self, cfg: dict, keep_k=None) -> _Config:
        c = _Config()
        for f in ("image_size", "patch_size", "in_chans", "tokens_in", "dim", "heads",
                  "mlp_hidden", "depth", "num_classes", "first_trainable", "loss"):
            setattr(c, f, int(cfg[f]))
        c.ln_eps = float(cfg.get("ln_eps", 1e-6))
        drops = list(cfg["drop_blocks"])
        c.n_drop = len(drops)
        n0 = (cfg["image_size"] // cfg["patch_size"]) ** 2 if cfg["image_size"] else cfg["tokens_in"] - 1
        if keep_k is None:
            keep_k = cfg.get("keep_k") or token_schedule(n0, cfg["keep_ratio"], len(drops),
                                                         bool(cfg.get("fuse_dropped")))
        for i, (b, k) in enumerate(zip(drops, keep_k)):
            c.drop_blocks[i] = b
            c.keep_k[i] = k
        c.fuse_dropped = int(bool(cfg.get("fuse_dropped")))
        c.n_experts = int(cfg.get("n_experts", 0))
        c.moe_top_k = int(cfg.get("moe_top_k", 0))
        for l in cfg.get("moe_blocks", ()):
            c.moe_block[l] = 1
        return c

    def _params(self, tensors: dict, keep: list) -> _Params:
        p = _Params()
        for name, a in tensors.items():
            if a is None:
                continue
            a = self.arr(a)
            keep.append(a)
            tensors[name] = a
            if name.startswith("blocks."):
                _, i, leaf = name.split(".")
                setattr(p.blocks[int(i)], leaf, a.ctypes.data)
            else:
                setattr(p, name, a.ctypes.data)
        return p

    # ---- the whole step ----------------------------------------------------------------
    def step(self, cfg: dict, params: dict, x, labels, forced_idx=None, want_grads=True,
             want_dx=False, keep_k=None, forced_experts=None) -> dict:
        """Run orc_step_moe.  Returns a dict with kept_idx (list per drop of [B,k]), scores (list per
        drop of [B,n]), x_trainable, x_final, logits, loss, grads (dict name -> array for the
        trainable tensors), dx_trainable when want_dx and, for mixture-of-experts blocks, experts
        (dict block -> [B*T,K]) and router_logits (dict block -> [B*T,E])."""
        c = self._config(cfg, keep_k)
        x = self.arr(x)
        B = x.shape[0]
        labels = np.ascontiguousarray(labels, dtype=np.int32)
        D, L, Cn = cfg["dim"], cfg["depth"], cfg["num_classes"]
        T0 = x.shape[1] if cfg["image_size"] == 0 else (cfg["image_size"] // cfg["patch_size"]) ** 2 + 1
        ks = [c.keep_k[i] for i in range(c.n_drop)]
        ns, n = [], T0 - 1
        T_at_block = []
        di = 0
        T = T0
        for l in range(L):
            T_at_block.append(T)
            if di < c.n_drop and c.drop_blocks[di] == l:
                ns.append(T - 1)
                T = ks[di] + 1 + (1 if c.fuse_dropped and T - 1 - ks[di] > 0 else 0)
                di += 1
        T_last = T
        moe = sorted(cfg.get("moe_blocks", ()))
        E, K = int(cfg.get("n_experts", 0)), int(cfg.get("moe_top_k", 0))
        Tm_at_block = [T_at_block[l + 1] if l + 1 < L else T_last for l in range(L)]   # tokens in the FFN
        m_rows = [B * Tm_at_block[l] for l in moe]
        ex_out = np.zeros(max(1, sum(m_rows) * max(K, 1)), dtype=np.int32)
        rl_out = np.zeros(max(1, sum(m_rows) * max(E, 1)), dtype=self.dtype)
        fex = None
        if forced_experts is not None:
            fex = np.ascontiguousarray(np.concatenate(
                [np.asarray(forced_experts[l], dtype=np.int32).reshape(-1) for l in moe]))
        ft = cfg["first_trainable"]
        T_f = T_at_block[ft] if ft < L else T_last
        keepalive = []
        p = self._params(dict(params), keepalive)
        kept = np.zeros(max(1, B * sum(ks)), dtype=np.int32)
        scores = np.zeros(max(1, B * sum(ns)), dtype=self.dtype)
        x_tr = np.zeros((B, T_f, D), dtype=self.dtype)
        x_fin = np.zeros((B, T_last, D), dtype=self.dtype)
        logits = np.zeros((B, max(Cn, 1)), dtype=self.dtype)
        loss = np.zeros(1, dtype=self.dtype)
        forced = None
        if forced_idx is not None:
            forced = np.ascontiguousarray(
                np.concatenate([np.asarray(f, dtype=np.int32).reshape(-1) for f in forced_idx])
                if len(forced_idx) else np.zeros(1, np.int32))
        grads = {}
        gp = None
        if want_grads:
            for name, a in params.items():
                tb = cfg.get("trainable_blocks")
                trainable = name in ("lnf_g", "lnf_b", "w_head", "b_head") or (
                    name.startswith("blocks.") and
                    ((int(name.split(".")[1]) in tb) if tb else int(name.split(".")[1]) >= ft))
                if trainable:
                    grads[name] = np.zeros(a.shape, dtype=self.dtype)
            gp = self._params(grads, keepalive)
        dx_tr = np.zeros((B, T_f, D), dtype=self.dtype) if (want_dx and want_grads) else None
        rc = self.lib.orc_step_moe(C.byref(c), C.byref(p), _ptr(x), _ptr(labels), C.c_int32(B),
                                   _ptr(forced), _ptr(x_tr), _ptr(kept), _ptr(scores), _ptr(x_fin),
                                   _ptr(logits), _ptr(loss), C.byref(gp) if gp is not None else None,
                                   _ptr(dx_tr), _ptr(fex), _ptr(ex_out), _ptr(rl_out))
        if rc != 0:
            raise ValueError(f"orc_step rejected the configuration (code {rc})")
        out_idx, out_sc, o1, o2 = [], [], 0, 0
        for k, n in zip(ks, ns):
            out_idx.append(kept[o1:o1 + B * k].reshape(B, k).copy())
            out_sc.append(scores[o2:o2 + B * n].reshape(B, n).copy())
            o1 += B * k
            o2 += B * n
        experts, router_logits, o1, o2 = {}, {}, 0, 0
        for l, m in zip(moe, m_rows):
            experts[l] = ex_out[o1:o1 + m * K].reshape(m, K).copy()
            router_logits[l] = rl_out[o2:o2 + m * E].reshape(m, E).copy()
            o1 += m * K
            o2 += m * E
        return dict(kept_idx=out_idx, scores=out_sc, x_trainable=x_tr, x_final=x_fin,
                    logits=logits if Cn else None, loss=float(loss[0]), grads=grads,
                    dx_trainable=dx_tr, keep_k=ks, tokens_per_block=T_at_block, T_last=T_last,
                    experts=experts, router_logits=router_logits)

    def adamw(self, w, g, m, v, lr, b1, b2, eps, wd, t):
        """In place on copies; returns (w, m, v)."""
        w, g, m, v = (self.arr(a).copy() for a in (w, g, m, v))
        self.lib.orc_adamw(_ptr(w), _ptr(g), _ptr(m), _ptr(v), C.c_int64(w.size), C.c_double(lr), C.c_double(b1),
                           C.c_double(b2), C.c_double(eps), C.c_double(wd), C.c_int32(t))
        return w, m, v

    # ---- mixture-of-experts FFN, for pins ----------------------------------------------
    def moe_route(self, logits, K, forced=None):
        logits = self.arr(logits); M, E = logits.shape
        ex = np.empty((M, K), np.int32); gates = np.empty((M, K), self.dtype)
        f = None if forced is None else np.ascontiguousarray(forced, dtype=np.int32)
        self.lib.orc_moe_route(_ptr(logits), C.c_int64(M), C.c_int32(E), C.c_int32(K), _ptr(f), _ptr(ex), _ptr(gates))
        return ex, gates

    def moe_ffn(self, h, w_router, w1, b1, w2, b2, K, forced=None):
        """Returns y and the saved tensors (dict) that moe_ffn_bwd takes."""
        h = self.arr(h); M, D = h.shape
        w_router, w1, b1, w2, b2 = (self.arr(a) for a in (w_router, w1, b1, w2, b2))
        E, _, F = w1.shape
        sv = dict(logits=np.empty((M, E), self.dtype), experts=np.empty((M, K), np.int32),
                  gates=np.empty((M, K), self.dtype), u=np.empty((M, K, F), self.dtype),
                  g=np.empty((M, K, F), self.dtype), ye=np.empty((M, K, D), self.dtype))
        y = np.empty((M, D), self.dtype)
        f = None if forced is None else np.ascontiguousarray(forced, dtype=np.int32)
        self.lib.orc_moe_ffn(_ptr(h), C.c_int64(M), C.c_int32(D), C.c_int32(F), C.c_int32(E), C.c_int32(K),
                             _ptr(w_router), _ptr(w1), _ptr(b1), _ptr(w2), _ptr(b2), _ptr(f), _ptr(sv["logits"]),
                             _ptr(sv["experts"]), _ptr(sv["gates"]), _ptr(sv["u"]), _ptr(sv["g"]), _ptr(sv["ye"]), _ptr(y))
        return y, sv

    def moe_ffn_bwd(self, dy, h, w_router, w1, w2, sv):
        dy = self.arr(dy); h = self.arr(h); M, D = h.shape
        w_router, w1, w2 = (self.arr(a) for a in (w_router, w1, w2))
        E, _, F = w1.shape
        K = sv["experts"].shape[1]
        dh = np.empty((M, D), self.dtype)
        g = dict(w_router=np.empty((D, E), self.dtype), w_fc1=np.empty((E, D, F), self.dtype),
                 b_fc1=np.empty((E, F), self.dtype), w_fc2=np.empty((E, F, D), self.dtype),
                 b_fc2=np.empty((E, D), self.dtype))
        self.lib.orc_moe_ffn_bwd(_ptr(dy), _ptr(h), C.c_int64(M), C.c_int32(D), C.c_int32(F), C.c_int32(E), C.c_int32(K),
                                 _ptr(w_router), _ptr(w1), _ptr(w2), _ptr(sv["experts"]), _ptr(sv["gates"]),
                                 _ptr(sv["u"]), _ptr(sv["g"]), _ptr(sv["ye"]), _ptr(dh), _ptr(g["w_router"]),
                                 _ptr(g["w_fc1"]), _ptr(g["b_fc1"]), _ptr(g["w_fc2"]), _ptr(g["b_fc2"]))
        return dh, g

    # ---- single layers, for pins -------------------------------------------------------
    def layernorm(self, x, gamma, beta, eps=1e-6):
        x = self.arr(x); M, D = x.shape
        y = np.empty_like(x); xhat = np.empty_like(x); rstd = np.empty(M, self.dtype)
        self.lib.orc_layernorm(_ptr(x), C.c_int64(M), C.c_int32(D), _ptr(self.arr(gamma)),
                               _ptr(self.arr(beta)), C.c_double(eps), _ptr(y), _ptr(xhat), _ptr(rstd))
        return y, xhat, rstd

    def layernorm_bwd(self, dy, xhat, rstd, gamma):
        dy = self.arr(dy); M, D = dy.shape
        dx = np.empty_like(dy); dg = np.empty(D, self.dtype); db = np.empty(D, self.dtype)
        self.lib.orc_layernorm_bwd(_ptr(dy), _ptr(self.arr(xhat)), _ptr(self.arr(rstd)),
                                   _ptr(self.arr(gamma)), C.c_int64(M), C.c_int32(D), _ptr(dx),
                                   _ptr(dg), _ptr(db))
        return dx, dg, db

    def linear(self, x, w, b):
        x = self.arr(x); w = self.arr(w); M, K = x.shape; N = w.shape[1]
        y = np.empty((M, N), self.dtype)
        self.lib.orc_linear(_ptr(x), C.c_int64(M), C.c_int32(K), _ptr(w),
                            _ptr(self.arr(b)) if b is not None else None, C.c_int32(N), _ptr(y))
        return y

    def linear_dgrad(self, dy, w):
        dy = self.arr(dy); w = self.arr(w); M, N = dy.shape; K = w.shape[0]
        dx = np.empty((M, K), self.dtype)
        self.lib.orc_linear_dgrad(_ptr(dy), C.c_int64(M), C.c_int32(N), _ptr(w), C.c_int32(K), _ptr(dx))
        return dx

    def linear_wgrad(self, x, dy):
        x = self.arr(x); dy = self.arr(dy); M, K = x.shape; N = dy.shape[1]
        dw = np.empty((K, N), self.dtype); db = np.empty(N, self.dtype)
        self.lib.orc_linear_wgrad(_ptr(x), _ptr(dy), C.c_int64(M), C.c_int32(K), C.c_int32(N),
                                  _ptr(dw), _ptr(db))
        return dw, db

    def attention(self, qkv, heads):
        qkv = self.arr(qkv); B, T, D3 = qkv.shape; D = D3 // 3
        P = np.empty((B, heads, T, T), self.dtype); o = np.empty((B, T, D), self.dtype)
        self.lib.orc_attention(_ptr(qkv), C.c_int32(B), C.c_int32(T), C.c_int32(heads),
                               C.c_int32(D // heads), _ptr(P), _ptr(o))
        return P, o

    def attention_bwd(self, qkv, P, dout, heads):
        qkv = self.arr(qkv); B, T, D3 = qkv.shape; D = D3 // 3
        dqkv = np.empty_like(qkv)
        self.lib.orc_attention_bwd(_ptr(qkv), _ptr(self.arr(P)), _ptr(self.arr(dout)), C.c_int32(B),
                                   C.c_int32(T), C.c_int32(heads), C.c_int32(D // heads), _ptr(dqkv))
        return dqkv

    def gelu(self, u):
        u = self.arr(u); g = np.empty_like(u)
        self.lib.orc_gelu(_ptr(u), C.c_int64(u.size), _ptr(g))
        return g

    def gelu_bwd(self, dg, u):
        u = self.arr(u); dg = self.arr(dg); du = np.empty_like(u)
        self.lib.orc_gelu_bwd(_ptr(dg), _ptr(u), C.c_int64(u.size), _ptr(du))
        return du

    def cls_scores(self, P):
        P = self.arr(P); B, H, T, _ = P.shape
        a = np.empty((B, T - 1), self.dtype)
        self.lib.orc_cls_scores(_ptr(P), C.c_int32(B), C.c_int32(H), C.c_int32(T), _ptr(a))
        return a

    def topk(self, a, k):
        a = self.arr(a).reshape(-1); idx = np.empty(max(k, 1), np.int32)
        self.lib.orc_topk(_ptr(a), C.c_int32(a.size), C.c_int32(k), _ptr(idx))
        return idx[:k]

    def gather(self, x, idx):
        x = self.arr(x); B, T, D = x.shape
        idx = np.ascontiguousarray(idx, np.int32); k = idx.shape[1]
        y = np.empty((B, k + 1, D), self.dtype)
        self.lib.orc_gather(_ptr(x), C.c_int32(B), C.c_int32(T), C.c_int32(D), _ptr(idx), C.c_int32(k), _ptr(y))
        return y

    def gather_bwd(self, dy, idx, T):
        dy = self.arr(dy); B, k1, D = dy.shape
        idx = np.ascontiguousarray(idx, np.int32)
        dx = np.empty((B, T, D), self.dtype)
        self.lib.orc_gather_bwd(_ptr(dy), C.c_int32(B), C.c_int32(T), C.c_int32(D), _ptr(idx),
                                C.c_int32(k1 - 1), _ptr(dx))
        return dx

    def stem(self, img, patch, w_patch, b_patch, cls, pos):
        img = self.arr(img); B, Ci, S, _ = img.shape; D = w_patch.shape[1]
        T = (S // patch) ** 2 + 1
        x = np.empty((B, T, D), self.dtype)
        self.lib.orc_stem(_ptr(img), C.c_int32(B), C.c_int32(Ci), C.c_int32(S), C.c_int32(patch),
                          C.c_int32(D), _ptr(self.arr(w_patch)), _ptr(self.arr(b_patch)),
                          _ptr(self.arr(cls)), _ptr(self.arr(pos)), _ptr(x))
        return x

    def cross_entropy(self, logits, labels):
        logits = self.arr(logits); B, Cn = logits.shape
        labels = np.ascontiguousarray(labels, np.int32)
        d = np.empty_like(logits)
        loss = self.lib.orc_cross_entropy(_ptr(logits), _ptr(labels), C.c_int32(B), C.c_int32(Cn), _ptr(d))
        return float(loss), d

    def sgd(self, w, g, m, lr, mu, wd):
        w = self.arr(w).copy(); g = self.arr(g)
        m = self.arr(m).copy() if m is not None else None
        self.lib.orc_sgd(_ptr(w), _ptr(g), _ptr(m), C.c_int64(w.size), C.c_double(lr),
                         C.c_double(mu), C.c_double(wd))
        return w, m
