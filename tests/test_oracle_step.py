"""Pins for the whole-step oracle: an independent PyTorch-CPU autograd composition, central finite
differences, the keep-ratio-1.0 identity, gradient-stop and dropped-token properties, and the
bookkeeping numbers the paper prints."""
import json
import os

import numpy as np
import pytest

import bsr_synth as S
from oracle import token_schedule
from oracle import accounting as acc

import torch_reference

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))


def rel(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300))


def setup(name, seed=0, std=0.02, **over):
    cfg = S.get_config(name, **over)
    p = S.make_params(cfg, seed=seed, std=std, bf16_exact=False)
    x, y = S.make_inputs(cfg, seed=seed, bf16_exact=False)
    return cfg, p, x, y


# ------------------------------------------------------------------ bookkeeping the paper prints

def test_token_schedule_pins():
    g = GOLD["drop_half_tokens"]
    assert token_schedule(g["n0"], 0.5, 3) == g["kept"]            # N/2, N/4, N/8
    assert token_schedule(196, 0.7, 3) == [137, 95, 66]
    assert token_schedule(64, 0.7, 1) == [44]
    assert token_schedule(196, 1.0, 3) == [196, 196, 196]
    assert token_schedule(100, 0.29, 1) == [29]                     # 0.29*100 = 28.999999999999996


def test_table1_saved_activation_bytes():
    MB = 1024.0 * 1024.0
    nl = acc.saved_bytes_nonlinear(T=197, D=384, H=6, F=1536)
    t1 = GOLD["table1_deit_s_b1_MB"]
    for key in ("qkv", "softmax_in", "gelu_in"):
        assert abs(nl[key] / MB - t1[key]) < 0.006, key             # printed to 2 decimals
    tot = GOLD["block_totals_MB"]
    assert abs(sum(nl.values()) / MB - tot["frozen_in_path"]) < 0.05
    assert abs(acc.saved_bytes_trainable(197, 384, 6, 1536) / MB - tot["trainable"]) < 0.05


def test_forward_macs_pins():
    g = GOLD["gmacs_b128"]
    full = lambda D, F: acc.forward_macs(acc.tokens_per_block(197, 12, [], []), D, F, 196, 768, 1000)
    assert abs(128 * full(384, 1536) / 1e9 - g["deit_s_full"]) < 1.0
    assert abs(128 * full(768, 3072) / 1e9 - g["vit_b_full"]) < 2.0
    assert abs(full(384, 1536) / 1e9 - GOLD["gmacs_b1_deit_s"]["value"]) < 0.05
    ks = token_schedule(196, 0.5, 3)
    tb = acc.tokens_per_block(197, 12, [3, 6, 9], ks)
    assert tb[3] == (197, 99) and tb[7] == (50, 50) and tb[11] == (25, 25)
    bsr_s = 128 * acc.forward_macs(tb, 384, 1536, 196, 768, 1000) / 1e9
    bsr_b = 128 * acc.forward_macs(tb, 768, 3072, 196, 768, 1000) / 1e9
    assert abs(bsr_s / g["deit_s_bsr"] - 1) < 0.02 and abs(bsr_b / g["vit_b_bsr"] - 1) < 0.02
    # Table 8: "drop rate" is the fraction dropped at each location
    for rate, drops, gmacs in GOLD["table8_gmacs"]["rows"]:
        tb = acc.tokens_per_block(197, 12, drops, token_schedule(196, 1.0 - rate, len(drops)))
        assert abs(128 * acc.forward_macs(tb, 384, 1536, 196, 768, 1000) / 1e9 / gmacs - 1) < 0.05


# ------------------------------------------------------------------ whole step vs torch autograd

@pytest.mark.parametrize("name", ["tiny_2blk", "mini_4blk", "c1_block_fp32"])
def test_step_matches_torch_autograd(orc64, name):
    cfg, p, x, y = setup(name, std=0.08)
    r = orc64.step(cfg, p, x, y, want_dx=True)
    t = torch_reference.run(cfg, p, x, y, r["kept_idx"])
    assert abs(r["loss"] - t["loss"]) < 1e-12 * max(1, abs(t["loss"]))
    assert rel(r["x_final"], t["x_final"]) < 1e-12
    if cfg["num_classes"]:
        assert rel(r["logits"], t["logits"]) < 1e-12
    for s_o, s_t in zip(r["scores"], t["scores"]):
        assert rel(s_o, s_t) < 1e-12
    assert rel(r["x_trainable"], t["x_trainable"]) < 1e-12
    assert rel(r["dx_trainable"], t["dx_trainable"]) < 1e-10
    assert set(r["grads"]) == set(t["grads"])
    for n in t["grads"]:
        assert rel(r["grads"][n], t["grads"][n]) < 1e-10, n
    # frozen tensors (stem, blocks before first_trainable) have no gradient entry at all
    for n in t["untouched"]:
        assert n not in r["grads"]


def test_kept_indices_follow_scores(orc64):
    cfg, p, x, y = setup("mini_4blk", std=0.2)
    r = orc64.step(cfg, p, x, y, want_grads=False)
    for sc, idx, k in zip(r["scores"], r["kept_idx"], r["keep_k"]):
        for b in range(sc.shape[0]):
            ref = np.sort(np.argsort(-sc[b], kind="stable")[:k])
            assert list(idx[b]) == list(ref)


def test_float32_oracle_agrees_with_float64(orc64, orc32):
    cfg, p, x, y = setup("mini_4blk", std=0.05)
    r64 = orc64.step(cfg, p, x, y)
    r32 = orc32.step(cfg, p, x, y, forced_idx=r64["kept_idx"])
    assert rel(r32["logits"], r64["logits"]) < 1e-5
    for n in r64["grads"]:
        assert rel(r32["grads"][n], r64["grads"][n]) < 1e-4, n


# ------------------------------------------------------------------ finite differences (Eq. 2-5)

@pytest.mark.parametrize("name", ["tiny_2blk", "c1_block_fp32"])
def test_finite_differences(orc64, name):
    over = dict(batch=2) if name == "tiny_2blk" else dict(dim=48, heads=3, mlp_hidden=96, tokens_in=17)
    cfg, p, x, y = setup(name, std=0.15, **over)
    base = orc64.step(cfg, p, x, y)
    idx = base["kept_idx"]
    g = np.random.default_rng(3)
    h = 1e-5
    for n, grad in base["grads"].items():
        flat = grad.reshape(-1)
        for j in g.choice(flat.size, size=min(3, flat.size), replace=False):
            q = {k: v.astype(np.float64).copy() for k, v in p.items()}
            q[n].reshape(-1)[j] += h
            lp = orc64.step(cfg, q, x, y, forced_idx=idx, want_grads=False)["loss"]
            q[n].reshape(-1)[j] -= 2 * h
            lm = orc64.step(cfg, q, x, y, forced_idx=idx, want_grads=False)["loss"]
            fd = (lp - lm) / (2 * h)
            assert abs(fd - flat[j]) <= 1e-6 * max(abs(fd), np.max(np.abs(flat)), 1e-8), (n, j, fd, flat[j])


# ------------------------------------------------------------------ properties of the method

def test_keep_ratio_one_is_the_undropped_model_bit_for_bit(orc64, orc32):
    for orc in (orc64, orc32):
        cfg, p, x, y = setup("mini_4blk")
        a = orc.step(dict(cfg, keep_ratio=1.0), p, x, y)
        b = orc.step(dict(cfg, drop_blocks=[]), p, x, y)
        assert a["keep_k"] == [64, 64]
        assert np.array_equal(a["logits"], b["logits"]) and a["loss"] == b["loss"]
        for n in b["grads"]:
            assert np.array_equal(a["grads"][n], b["grads"][n]), n


def test_gradient_stops_at_the_first_trainable_block(orc64):
    cfg, p, x, y = setup("mini_4blk", std=0.1)
    r = orc64.step(cfg, p, x, y)
    names = set(r["grads"])
    assert all(not n.startswith(("blocks.0.", "blocks.1.", "w_patch", "b_patch", "cls", "pos")) for n in names)
    assert {"blocks.2.w_qkv", "blocks.3.ln2_b", "lnf_g", "w_head", "b_head"} <= names
    # a frozen weight influences trainable gradients only through the forward activations:
    # feeding the same x_trainable through a model whose frozen part differs gives the same grads
    cfg_t = dict(cfg, image_size=0, tokens_in=r["x_trainable"].shape[1], depth=2, first_trainable=0,
                 drop_blocks=[0], keep_k=[r["keep_k"][1]])
    p_t = {n.replace("blocks.2.", "blocks.0.").replace("blocks.3.", "blocks.1."): v
           for n, v in p.items() if n.startswith(("blocks.2.", "blocks.3.", "lnf", "w_head", "b_head"))}
    t = orc64.step(cfg_t, p_t, r["x_trainable"], y)
    assert np.array_equal(t["logits"], r["logits"])
    assert np.array_equal(t["grads"]["blocks.0.w_fc1"], r["grads"]["blocks.2.w_fc1"])


def test_dropped_tokens_get_gradient_only_through_keys_and_values(orc64):
    cfg, p, x, y = setup("c1_block_fp32", std=0.1)
    r = orc64.step(cfg, p, x, y, want_dx=True)
    T = cfg["tokens_in"]
    dropped = np.setdiff1d(np.arange(T - 1), r["kept_idx"][0][0]) + 1
    dx = r["dx_trainable"][0]
    assert np.all(np.abs(dx[dropped]).sum(axis=1) > 0)      # K/V path of the block's own attention
    # ... and through nothing else: with K = V = 0 a dropped token cannot influence the loss at all
    q = {k: v.copy() for k, v in p.items()}
    D = cfg["dim"]
    q["blocks.0.w_qkv"][:, D:] = 0
    q["blocks.0.b_qkv"][D:] = 0
    r2 = orc64.step(cfg, q, x, y, want_dx=True, forced_idx=r["kept_idx"])
    dx2 = r2["dx_trainable"][0]
    kept = r["kept_idx"][0][0] + 1
    assert np.all(dx2[dropped] == 0)
    assert np.all(np.abs(dx2[kept]).sum(axis=1) > 0) and np.abs(dx2[0]).sum() > 0


def test_permuting_patch_tokens_permutes_the_kept_set(orc64):
    cfg, p, x, y = setup("c1_block_fp32", std=0.1)
    r = orc64.step(cfg, p, x, y, want_grads=False)
    perm = np.random.default_rng(5).permutation(cfg["tokens_in"] - 1)
    xp = x.copy()
    xp[:, 1:] = x[:, 1 + perm]
    rp = orc64.step(cfg, p, xp, y, want_grads=False)
    for b in range(x.shape[0]):
        assert set(perm[rp["kept_idx"][0][b]]) == set(r["kept_idx"][0][b])
    # the CLS output only depends on the set of kept tokens
    assert rel(rp["x_final"][:, 0], r["x_final"][:, 0]) < 1e-12


def test_mean_square_loss_value(orc64):
    cfg, p, x, y = setup("c1_block_fp32")
    r = orc64.step(cfg, p, x, y, want_grads=False)
    assert r["x_final"].shape == (2, 45, 192)
    assert abs(r["loss"] - float(np.mean(r["x_final"] ** 2))) < 1e-14


def test_bad_configuration_is_rejected(orc64):
    cfg, p, x, y = setup("tiny_2blk")
    with pytest.raises(ValueError):
        orc64.step(dict(cfg, drop_blocks=[1, 0]), p, x, y, keep_k=[5, 3])
    with pytest.raises(ValueError):
        orc64.step(cfg, p, x, y, keep_k=[99])


# ------------------------------------------------------------------ interleaved trainable layout

def test_interleaved_layout_against_torch_and_finite_differences(orc64):
    """Trainable blocks {1,3,5} with frozen blocks between them (the paper's default layout, Sec. 5):
    the frozen blocks in the path pass the input gradient on and get no weight gradient."""
    cfg, p, x, y = setup("mini_interleaved")
    r = orc64.step(cfg, p, x, y, want_dx=True)
    t = torch_reference.run(cfg, p, x, y, r["kept_idx"])
    assert abs(r["loss"] - t["loss"]) < 1e-10
    names = set(r["grads"])
    assert names == set(t["grads"])
    assert not any(n.startswith(("blocks.0.", "blocks.2.", "blocks.4.")) for n in names)
    assert any(n.startswith("blocks.1.") for n in names) and any(n.startswith("blocks.5.") for n in names)
    for n in names:
        assert rel(r["grads"][n], t["grads"][n]) < 1e-8, n
    assert rel(r["dx_trainable"], t["dx_trainable"]) < 1e-8
    # central differences through the frozen blocks 2 and 4 into block 1
    eps = 1e-6
    for name, ix in (("blocks.1.w_fc1", (3, 5)), ("blocks.1.ln1_g", (7,)), ("blocks.3.w_qkv", (2, 9))):
        pp, pm = dict(p), dict(p)
        pp[name] = p[name].astype(np.float64).copy(); pp[name][ix] += eps
        pm[name] = p[name].astype(np.float64).copy(); pm[name][ix] -= eps
        lp = orc64.step(cfg, pp, x, y, forced_idx=r["kept_idx"], want_grads=False)["loss"]
        lm = orc64.step(cfg, pm, x, y, forced_idx=r["kept_idx"], want_grads=False)["loss"]
        fd = (lp - lm) / (2 * eps)
        assert abs(fd - r["grads"][name][ix]) < 1e-6 * max(1.0, abs(fd)), (name, fd, r["grads"][name][ix])


# ------------------------------------------------------------------ fused inattentive token

@pytest.mark.parametrize("name", ["tiny_2blk", "mini_4blk", "mini_interleaved"])
def test_fused_token_against_torch_and_properties(orc64, name):
    """Sec. 4.1: the dropped tokens are fused into one token (importance-weighted average) that follows
    the kept ones; weights and indices are constants of the backward pass."""
    cfg, p, x, y = setup(name, fuse_dropped=1)
    r = orc64.step(cfg, p, x, y, want_dx=True)
    t = torch_reference.run(cfg, p, x, y, r["kept_idx"])
    assert abs(r["loss"] - t["loss"]) < 1e-10
    for n in r["grads"]:
        assert rel(r["grads"][n], t["grads"][n]) < 1e-8, n
    assert rel(r["dx_trainable"], t["dx_trainable"]) < 1e-8
    plain = orc64.step(S.get_config(name), p, x, y, want_grads=False)
    assert r["T_last"] > plain["T_last"]
    if max(cfg["drop_blocks"]) < cfg["depth"] - 1:       # a later attention sees the fused token
        assert abs(r["loss"] - plain["loss"]) > 1e-12
    # token schedule: one extra patch token after every drop that drops something
    n0 = r["tokens_per_block"][0] - 1
    assert r["keep_k"] == token_schedule(n0, cfg["keep_ratio"], len(cfg["drop_blocks"]), fuse=True)
    # keep ratio 1.0: nothing is dropped, nothing is fused, identical to the plain model
    a = orc64.step(S.get_config(name, fuse_dropped=1, keep_ratio=1.0), p, x, y, want_grads=False)
    b = orc64.step(S.get_config(name, keep_ratio=1.0), p, x, y, want_grads=False)
    assert a["loss"] == b["loss"] and a["T_last"] == b["T_last"]


def test_fused_token_is_the_weighted_mean(orc64):
    rng = np.random.default_rng(0)
    B, T, D, k = 2, 9, 5, 3
    x = rng.standard_normal((B, T, D)); a = rng.random((B, T - 1)) + 0.1
    idx = np.stack([np.sort(rng.choice(T - 1, k, replace=False)) for _ in range(B)]).astype(np.int32)
    wts = np.zeros((B, T - 1)); f = np.zeros((B, D))
    import ctypes as C
    orc64.lib.orc_fuse_dropped(x.ctypes.data_as(C.c_void_p), a.ctypes.data_as(C.c_void_p), B, T, D,
                               idx.ctypes.data_as(C.c_void_p), k, wts.ctypes.data_as(C.c_void_p),
                               f.ctypes.data_as(C.c_void_p))
    for b in range(B):
        drop = [j for j in range(T - 1) if j not in idx[b]]
        want = np.average(x[b, 1:][drop], axis=0, weights=a[b, drop])       # numpy's weighted mean
        assert np.allclose(f[b], want, rtol=1e-12)
        assert np.allclose(wts[b].sum(), 1.0) and (wts[b, idx[b]] == 0).all()
    # equal dropped tokens fuse to that token, whatever the scores
    x[:, 1:] = x[:, 1:2]
    orc64.lib.orc_fuse_dropped(x.ctypes.data_as(C.c_void_p), a.ctypes.data_as(C.c_void_p), B, T, D,
                               idx.ctypes.data_as(C.c_void_p), k, wts.ctypes.data_as(C.c_void_p),
                               f.ctypes.data_as(C.c_void_p))
    assert np.allclose(f, x[:, 1], rtol=1e-12)


def test_fused_token_finite_differences(orc64):
    """Central differences for parameters downstream of the fusion (the fusion weights are constants
    of the method's backward pass, so parameters that move the scores are not probed)."""
    cfg, p, x, y = setup("mini_4blk", fuse_dropped=1)      # drops at blocks 1 and 2, trainable 2 and 3
    r = orc64.step(cfg, p, x, y)
    eps = 1e-6
    for name, ix in (("blocks.3.w_qkv", (2, 9)), ("blocks.3.w_fc1", (3, 5)), ("blocks.2.w_fc2", (4, 4))):
        pp, pm = dict(p), dict(p)
        pp[name] = p[name].astype(np.float64).copy(); pp[name][ix] += eps
        pm[name] = p[name].astype(np.float64).copy(); pm[name][ix] -= eps
        lp = orc64.step(cfg, pp, x, y, forced_idx=r["kept_idx"], want_grads=False)["loss"]
        lm = orc64.step(cfg, pm, x, y, forced_idx=r["kept_idx"], want_grads=False)["loss"]
        fd = (lp - lm) / (2 * eps)
        assert abs(fd - r["grads"][name][ix]) < 1e-6 * max(1.0, abs(fd)), (name, fd, r["grads"][name][ix])
