"""Pins for the mixture-of-experts FFN of the oracle (Sec. 5.3): brute-force routing on small inputs,
an independent PyTorch-CPU autograd composition (torch.topk, softmax, index_select / index_add), the
special case of identical experts (reduces to the dense FFN), central finite differences, and the
whole step against the torch composition."""
import numpy as np
import pytest
import torch

import bsr_synth as S
import torch_reference


def rel(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300))


def draw(rng, M=23, D=12, F=20, E=5):
    h = rng.standard_normal((M, D))
    wr = rng.standard_normal((D, E)) / np.sqrt(D)
    w1 = rng.standard_normal((E, D, F)) * 0.3
    b1 = rng.standard_normal((E, F)) * 0.1
    w2 = rng.standard_normal((E, F, D)) * 0.3
    b2 = rng.standard_normal((E, D)) * 0.1
    return h, wr, w1, b1, w2, b2


def test_route_brute_force_and_ties(orc64):
    rng = np.random.default_rng(0)
    for E, K in ((4, 1), (5, 2), (16, 2), (16, 4), (3, 3)):
        lg = rng.standard_normal((200, E))
        lg[::7] = np.round(lg[::7])              # rows full of ties
        lg[5] = 0.25                             # all equal: lowest indices win, in order
        ex, gates = orc64.moe_route(lg, K)
        for t in range(lg.shape[0]):
            order = sorted(range(E), key=lambda e: (-lg[t, e], e))[:K]      # the definition
            assert list(ex[t]) == order
            sel = lg[t, order]
            want = np.exp(sel - sel.max()) / np.exp(sel - sel.max()).sum()
            assert np.allclose(gates[t], want, rtol=1e-12, atol=0)
        assert np.allclose(gates.sum(axis=1), 1.0, atol=1e-14)
        assert (np.sort(ex, axis=1)[:, 1:] != np.sort(ex, axis=1)[:, :-1]).all()   # K distinct experts
    forced = np.array([[2, 0]] * 200, dtype=np.int32)
    ex, gates = orc64.moe_route(lg[:, :3].copy(), 2, forced=forced)
    assert (ex == forced).all()
    sel = np.take_along_axis(lg[:, :3], forced, axis=1)
    assert np.allclose(gates, np.exp(sel) / np.exp(sel).sum(axis=1, keepdims=True), rtol=1e-12)


@pytest.mark.parametrize("K", [1, 2, 4])
def test_moe_ffn_against_torch_autograd(orc64, K):
    rng = np.random.default_rng(10 + K)
    h, wr, w1, b1, w2, b2 = draw(rng)
    dy = rng.standard_normal(h.shape)
    y, sv = orc64.moe_ffn(h, wr, w1, b1, w2, b2, K)
    dh, g = orc64.moe_ffn_bwd(dy, h, wr, w1, w2, sv)
    T = {n: torch.tensor(a, dtype=torch.float64, requires_grad=True)
         for n, a in dict(h=h, wr=wr, w1=w1, b1=b1, w2=w2, b2=b2).items()}
    yt, ext = torch_reference.moe_ffn(T["h"], T["wr"], T["w1"], T["b1"], T["w2"], T["b2"], K)
    assert (np.sort(ext.numpy(), axis=1) == np.sort(sv["experts"], axis=1)).all()
    (yt * torch.tensor(dy)).sum().backward()
    assert rel(y, yt.detach().numpy()) < 1e-12
    assert rel(dh, T["h"].grad.numpy()) < 1e-11
    for name, key in (("w_router", "wr"), ("w_fc1", "w1"), ("b_fc1", "b1"), ("w_fc2", "w2"), ("b_fc2", "b2")):
        assert rel(g[name], T[key].grad.numpy()) < 1e-11, name
    # the expert outputs really are weighted: K = 1 has gate 1, larger K mixes
    if K == 1:
        assert np.allclose(sv["gates"], 1.0)


def test_identical_experts_reduce_to_the_dense_ffn(orc64):
    rng = np.random.default_rng(3)
    h, wr, w1, b1, w2, b2 = draw(rng, E=4)
    w1[:] = w1[0]; b1[:] = b1[0]; w2[:] = w2[0]; b2[:] = b2[0]
    y, _ = orc64.moe_ffn(h, wr, w1, b1, w2, b2, 2)
    u = orc64.linear(h, w1[0], b1[0])
    dense = orc64.linear(orc64.gelu(u), w2[0], b2[0])          # gates sum to one
    assert rel(y, dense) < 1e-13


def test_moe_ffn_finite_differences(orc64):
    rng = np.random.default_rng(5)
    h, wr, w1, b1, w2, b2 = draw(rng, M=9, D=6, F=7, E=4)
    dy = rng.standard_normal(h.shape)
    y, sv = orc64.moe_ffn(h, wr, w1, b1, w2, b2, 2)
    dh, g = orc64.moe_ffn_bwd(dy, h, wr, w1, w2, sv)
    forced = sv["experts"]

    def loss(**kw):
        a = dict(h=h, wr=wr, w1=w1, b1=b1, w2=w2, b2=b2); a.update(kw)
        yy, _ = orc64.moe_ffn(a["h"], a["wr"], a["w1"], a["b1"], a["w2"], a["b2"], 2, forced=forced)
        return float((yy * dy).sum())
    eps = 1e-6
    for key, grad, idxs in (("wr", g["w_router"], [(0, 0), (3, 2), (5, 1)]), ("h", dh, [(0, 0), (4, 3), (8, 5)]),
                            ("w1", g["w_fc1"], [(0, 0, 0), (2, 3, 4)]), ("b2", g["b_fc2"], [(1, 2), (3, 0)])):
        base = dict(h=h, wr=wr, w1=w1, b1=b1, w2=w2, b2=b2)[key]
        for ix in idxs:
            p, m = base.copy(), base.copy()
            p[ix] += eps; m[ix] -= eps
            fd = (loss(**{key: p}) - loss(**{key: m})) / (2 * eps)
            assert abs(fd - grad[ix]) <= 1e-6 * max(1.0, abs(fd)), (key, ix, fd, grad[ix])


@pytest.mark.parametrize("name", ["tiny_moe", "mini_moe"])
def test_step_with_moe_blocks_against_torch(orc64, name):
    cfg = S.get_config(name)
    p = S.make_params(cfg, bf16_exact=False)
    x, y = S.make_inputs(cfg, bf16_exact=False)
    r = orc64.step(cfg, p, x, y, want_dx=True)
    t = torch_reference.run(cfg, p, x, y, r["kept_idx"], experts=r["experts"])
    assert abs(r["loss"] - t["loss"]) < 1e-10
    assert rel(r["logits"], t["logits"]) < 1e-10
    assert set(r["grads"]) == set(t["grads"])
    for n in r["grads"]:
        assert rel(r["grads"][n], t["grads"][n]) < 1e-8, n
    assert rel(r["dx_trainable"], t["dx_trainable"]) < 1e-8
    # free-running torch.topk picks the same experts wherever the logit gap is clear
    t2 = torch_reference.run(cfg, p, x, y, r["kept_idx"])
    assert abs(r["loss"] - t2["loss"]) < 1e-9
    # the router and the used experts of a trainable mixture block receive gradient; an expert that no
    # token chose receives exactly none (in the last block only the CLS tokens reach the loss)
    for l in cfg["moe_blocks"]:
        if l >= cfg["first_trainable"]:
            assert np.abs(r["grads"][f"blocks.{l}.w_router"]).max() > 0
            per_expert = np.abs(r["grads"][f"blocks.{l}.w_fc1"]).reshape(cfg["n_experts"], -1).max(axis=1)
            assert (per_expert > 0).any()
            unused = sorted(set(range(cfg["n_experts"])) - set(r["experts"][l].reshape(-1).tolist()))
            assert (per_expert[unused] == 0).all()


def test_forced_experts_are_used(orc64):
    cfg = S.get_config("tiny_moe")
    p = S.make_params(cfg, bf16_exact=False)
    x, y = S.make_inputs(cfg, bf16_exact=False)
    r = orc64.step(cfg, p, x, y, want_grads=False)
    forced = {l: (e[:, ::-1].copy() + 1) % cfg["n_experts"] for l, e in r["experts"].items()}
    r2 = orc64.step(cfg, p, x, y, want_grads=False, forced_experts=forced)
    for l in forced:
        assert (r2["experts"][l] == forced[l]).all()
    assert abs(r2["loss"] - r["loss"]) > 1e-9
