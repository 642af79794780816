"""Pins for the single layers of the CPU oracle: each one against a numpy / torch-CPU library
routine, a closed form, or an invariant.  A dropped term, a wrong sign or a transposed operand in
the oracle fails at least one of these."""
import itertools
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

rng = np.random.default_rng(7)


def close(a, b, tol=1e-10):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return np.max(np.abs(a - b)) <= tol * max(1.0, np.max(np.abs(b)))


def test_layernorm_matches_torch(orc64):
    x = rng.standard_normal((7, 33)) * 3 + 1.5
    g = 1 + 0.1 * rng.standard_normal(33)
    b = 0.1 * rng.standard_normal(33)
    y, xhat, rstd = orc64.layernorm(x, g, b, 1e-6)
    ref = F.layer_norm(torch.tensor(x), (33,), torch.tensor(g), torch.tensor(b), 1e-6).numpy()
    assert close(y, ref)
    assert close(xhat.mean(axis=1), 0 * rstd, 1e-12)
    assert close((xhat ** 2).mean(axis=1), 1 - 1e-6 * rstd ** 2, 1e-10)  # biased variance + eps


def test_layernorm_bwd_matches_autograd(orc64):
    x = torch.tensor(rng.standard_normal((9, 20)), requires_grad=True)
    g = torch.tensor(1 + 0.1 * rng.standard_normal(20), requires_grad=True)
    b = torch.tensor(0.1 * rng.standard_normal(20), requires_grad=True)
    dy = rng.standard_normal((9, 20))
    F.layer_norm(x, (20,), g, b, 1e-6).backward(torch.tensor(dy))
    _, xhat, rstd = orc64.layernorm(x.detach().numpy(), g.detach().numpy(), b.detach().numpy())
    dx, dg, db = orc64.layernorm_bwd(dy, xhat, rstd, g.detach().numpy())
    assert close(dx, x.grad.numpy()) and close(dg, g.grad.numpy()) and close(db, b.grad.numpy())


def test_linear_forward_and_eq2_eq4(orc64):
    # rectangular shapes so that a transposed operand cannot pass
    x = rng.standard_normal((11, 5)); w = rng.standard_normal((5, 8)); b = rng.standard_normal(8)
    dy = rng.standard_normal((11, 8))
    assert close(orc64.linear(x, w, b), x @ w + b)
    assert close(orc64.linear(x, w, None), x @ w)
    assert close(orc64.linear_dgrad(dy, w), dy @ w.T)          # Eq. 2
    dw, db = orc64.linear_wgrad(x, dy)
    assert close(dw, x.T @ dy) and close(db, dy.sum(axis=0))   # Eq. 4


def _split_heads(qkv, H):
    B, T, D3 = qkv.shape
    D = D3 // 3
    t = torch.tensor(qkv).reshape(B, T, 3, H, D // H).permute(2, 0, 3, 1, 4)
    return t[0], t[1], t[2]


def test_attention_matches_sdpa_and_rows_sum_to_one(orc64):
    B, T, H, d = 2, 13, 3, 8
    qkv = rng.standard_normal((B, T, 3 * H * d))
    P, o = orc64.attention(qkv, H)
    assert np.max(np.abs(P.sum(axis=-1) - 1)) < 1e-12
    assert P.min() > 0
    q, k, v = _split_heads(qkv, H)
    ref = F.scaled_dot_product_attention(q, k, v).transpose(1, 2).reshape(B, T, H * d).numpy()
    assert close(o, ref)
    refP = torch.softmax(q @ k.transpose(-1, -2) / math.sqrt(d), -1).numpy()   # Eq. 1
    assert close(P, refP)


def test_attention_float32_rows_sum_to_one(orc32):
    qkv = rng.standard_normal((2, 65, 3 * 192)).astype(np.float32)
    P, _ = orc32.attention(qkv, 3)
    assert np.max(np.abs(P.sum(axis=-1, dtype=np.float64) - 1)) < 1e-6


def test_attention_bwd_matches_autograd(orc64):
    B, T, H, d = 2, 9, 2, 4
    qkv = torch.tensor(rng.standard_normal((B, T, 3 * H * d)), requires_grad=True)
    t = qkv.reshape(B, T, 3, H, d).permute(2, 0, 3, 1, 4)
    o = F.scaled_dot_product_attention(t[0], t[1], t[2]).transpose(1, 2).reshape(B, T, H * d)
    do = rng.standard_normal((B, T, H * d))
    o.backward(torch.tensor(do))
    P, _ = orc64.attention(qkv.detach().numpy(), H)
    dqkv = orc64.attention_bwd(qkv.detach().numpy(), P, do, H)
    assert close(dqkv, qkv.grad.numpy())


def test_gelu_is_exact_erf_form(orc64):
    u = np.concatenate([rng.standard_normal(200) * 3, [0.0, -8.0, 8.0]])
    assert close(orc64.gelu(u), F.gelu(torch.tensor(u)).numpy(), 1e-14)   # approximate='none'
    # closed form at a few points: GELU(x) = x * Phi(x)
    assert abs(orc64.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15
    ut = torch.tensor(u, requires_grad=True)
    dg = rng.standard_normal(u.shape)
    F.gelu(ut).backward(torch.tensor(dg))
    assert close(orc64.gelu_bwd(dg, u), ut.grad.numpy(), 1e-13)


def test_cls_scores_head_mean_and_mass(orc64):
    B, T, H, d = 3, 10, 4, 4
    P, _ = orc64.attention(rng.standard_normal((B, T, 3 * H * d)), H)
    a = orc64.cls_scores(P)
    assert a.shape == (B, T - 1)
    assert close(a, P[:, :, 0, 1:].mean(axis=1))
    # the CLS column takes part in the softmax but not in the ranking
    assert close(a.sum(axis=1), 1 - P[:, :, 0, 0].mean(axis=1))


def test_head_mean_of_probabilities_is_not_mean_of_logits(orc64):
    # With H > 1, averaging softmax rows and averaging logits rank tokens differently; the reading
    # taken for Eq. 6 is the head mean of the post-softmax CLS row.
    H, d, T = 2, 1, 4
    qkv = np.zeros((1, T, 3 * H * d))
    qkv[0, 0, 0:2] = [1.0, 1.0]                    # CLS query of head 0 / head 1
    k0, k1 = [10.0, 9.0, 0.0], [0.0, 2.0, 6.0]     # patch keys per head (CLS key = 0)
    qkv[0, 1:, 2] = k0
    qkv[0, 1:, 3] = k1
    P, _ = orc64.attention(qkv, H)
    a = orc64.cls_scores(P)[0]
    p0 = np.exp([0.0] + k0); p0 /= p0.sum()
    p1 = np.exp([0.0] + k1); p1 /= p1.sum()
    assert close(a, (p0[1:] + p1[1:]) / 2)
    assert int(np.argmax((np.array(k0) + np.array(k1)) / 2)) == 1   # mean of logits would pick 1
    assert list(orc64.topk(a, 1)) == [2]                             # mean of probabilities picks 2


@pytest.mark.parametrize("n,k", [(1, 0), (1, 1), (5, 2), (8, 8), (9, 4), (12, 7)])
def test_topk_brute_force(orc64, n, k):
    for trial in range(20):
        a = rng.integers(0, 4, n).astype(np.float64) if trial % 2 else rng.standard_normal(n)
        idx = list(orc64.topk(a, k))
        assert idx == sorted(idx) and len(set(idx)) == k
        best = max(sum(a[list(s)]) for s in itertools.combinations(range(n), k))
        assert abs(sum(a[idx]) - best) < 1e-12
        # among all optimal subsets the tie rule (lower index first) picks the lexicographically smallest
        opt = [s for s in itertools.combinations(range(n), k) if abs(sum(a[list(s)]) - best) < 1e-12]
        assert tuple(idx) == min(opt)


def test_topk_vs_stable_sort_and_ties(orc64):
    for n, k in [(196, 137), (137, 95), (95, 66), (64, 44), (196, 98)]:
        a = np.round(rng.standard_normal(n), 1)          # many exact ties
        ref = np.sort(np.argsort(-a, kind="stable")[:k])
        assert list(orc64.topk(a, k)) == list(ref)
    assert list(orc64.topk(np.ones(10), 4)) == [0, 1, 2, 3]
    assert list(orc64.topk(np.arange(10.0), 3)) == [7, 8, 9]


def test_gather_and_its_adjoint(orc64):
    B, T, D, k = 3, 9, 4, 5
    x = rng.standard_normal((B, T, D))
    idx = np.stack([np.sort(rng.choice(T - 1, k, replace=False)) for _ in range(B)]).astype(np.int32)
    y = orc64.gather(x, idx)
    for b in range(B):
        assert np.array_equal(y[b, 0], x[b, 0])
        assert np.array_equal(y[b, 1:], x[b, 1 + idx[b]])
    dy = rng.standard_normal(y.shape)
    dx = orc64.gather_bwd(dy, idx, T)
    assert abs((dx * x).sum() - (dy * y).sum()) < 1e-10          # <G^T dy, x> = <dy, G x>
    dropped = np.setdiff1d(np.arange(T - 1), idx[0]) + 1
    assert np.all(dx[0, dropped] == 0)
    full = np.tile(np.arange(T - 1, dtype=np.int32), (B, 1))
    assert np.array_equal(orc64.gather(x, full), x)               # keeping everything is the identity


def test_stem_is_a_strided_convolution(orc64):
    B, C, S, p, D = 2, 3, 12, 4, 10
    img = rng.standard_normal((B, C, S, S))
    w = rng.standard_normal((C * p * p, D)); b = rng.standard_normal(D)
    cls = rng.standard_normal(D); pos = rng.standard_normal(((S // p) ** 2 + 1, D))
    x = orc64.stem(img, p, w, b, cls, pos)
    conv = F.conv2d(torch.tensor(img), torch.tensor(w.T.reshape(D, C, p, p).copy()), torch.tensor(b),
                    stride=p).flatten(2).transpose(1, 2).numpy()
    assert close(x[:, 1:], conv + pos[1:])
    assert close(x[:, 0], np.tile(cls + pos[0], (B, 1)))


def test_cross_entropy_matches_torch(orc64):
    z = rng.standard_normal((6, 11)) * 4
    y = rng.integers(0, 11, 6)
    zt = torch.tensor(z, requires_grad=True)
    ref = F.cross_entropy(zt, torch.tensor(y))
    ref.backward()
    loss, d = orc64.cross_entropy(z, y)
    assert abs(loss - float(ref.detach())) < 1e-12 and close(d, zt.grad.numpy())
    assert np.max(np.abs(d.sum(axis=1))) < 1e-15


def test_sgd_closed_form(orc64):
    w, _ = orc64.sgd(np.array([2.0]), np.array([0.5]), None, lr=0.1, mu=0.0, wd=0.0)
    assert abs(w[0] - 1.95) < 1e-15
    w, _ = orc64.sgd(np.array([2.0]), np.array([0.5]), None, lr=0.1, mu=0.0, wd=0.25)
    assert abs(w[0] - (2 - 0.1 * (0.5 + 0.5))) < 1e-15
    # two momentum steps against torch.optim.SGD
    wt = torch.tensor([1.0, -2.0, 3.0], dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([wt], lr=0.05, momentum=0.9, weight_decay=1e-2)
    w = wt.detach().numpy().copy(); m = np.zeros(3)
    for g in ([0.3, -0.1, 0.2], [0.1, 0.4, -0.5]):
        wt.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, m = orc64.sgd(w, np.array(g), m, lr=0.05, mu=0.9, wd=1e-2)
    assert close(w, wt.detach().numpy(), 1e-14)


def test_adamw_against_torch_optimizer(orc64):
    """orc_adamw against torch.optim.AdamW (decoupled weight decay), three steps."""
    import torch
    rng = np.random.default_rng(4)
    w0 = rng.standard_normal(257); gs = [rng.standard_normal(257) for _ in range(3)]
    lr, b1, b2, eps, wd = 3e-3, 0.9, 0.98, 1e-8, 0.05
    p = torch.tensor(w0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([p], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    w, m, v = w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
    for t, g in enumerate(gs, 1):
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, m, v = orc64.adamw(w, g, m, v, lr, b1, b2, eps, wd, t)
        assert np.allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-14), t
    assert np.abs(w - w0).max() > 1e-3
