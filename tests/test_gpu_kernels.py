"""Kernel-level GPU parity: the bf16 MFMA GEMMs at the real shapes of the ViT-B/16 workload
(M = B*T in {6304, 4416, 3072, 2144}, widths 768 / 2304 / 3072) plus ragged sizes, against the
oracle's linear layers on sampled rows (rows of a linear layer are independent)."""
import numpy as np
import pytest

import bsr_synth as S

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device")
    import paper_2405_10951_amd as P
    return torch, P


def bf16_np(rng, shape, scale=1.0):
    return S.round_to_bf16((rng.standard_normal(shape) * scale).astype(np.float32))


def to_dev(torch, a, dtype=None):
    t = torch.as_tensor(a).cuda()
    return t.to(dtype) if dtype is not None else t


def assert_close(got, ref, what, tol=1e-2):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    err = np.abs(got - ref)
    assert err.max() <= tol * np.abs(ref).max(), f"{what}: max err {err.max():.3g} vs max {np.abs(ref).max():.3g}"
    rms = np.sqrt(np.mean(ref ** 2))
    bad = err > tol * np.abs(ref) + tol * rms
    assert bad.mean() < 1e-4, f"{what}: {bad.mean():.2%} elements outside tolerance"


SHAPES = [(6304, 768, 2304), (4416, 768, 768), (3072, 768, 3072), (2144, 3072, 768),
          (2144, 768, 2304), (333, 200, 72), (1, 64, 8), (130, 776, 136)]


@pytest.mark.parametrize("M,kin,out", SHAPES)
def test_linear_forward(env, orc64, M, kin, out):
    torch, P = env
    rng = np.random.default_rng(M + kin + out)
    x = bf16_np(rng, (M, kin)); w = bf16_np(rng, (kin, out), 0.05); b = rng.standard_normal(out).astype(np.float32)
    res = bf16_np(rng, (M, out))
    rows = np.unique(np.concatenate([rng.choice(M, min(M, 192), replace=False), np.arange(max(0, M - 40), M)]))
    xt = to_dev(torch, x, torch.bfloat16)
    wt = to_dev(torch, np.ascontiguousarray(w.T), torch.bfloat16)
    bt = to_dev(torch, b)
    # plain: y = x W + b
    y, used = P.bsr_linear_forward(xt, wt, bt)
    torch.cuda.synchronize()
    ref = orc64.linear(x[rows], w, b)
    assert used == 1, "the MFMA kernel must take this shape"
    assert_close(y.float().cpu().numpy()[rows], ref, "linear")
    # GELU epilogue with the stored pre-activation, and the residual epilogue
    u = torch.empty((M, out), dtype=torch.bfloat16, device="cuda")
    g, _ = P.bsr_linear_forward(xt, wt, bt, act=1, u_out=u)
    r, _ = P.bsr_linear_forward(xt, wt, bt, res=to_dev(torch, res, torch.bfloat16))
    torch.cuda.synchronize()
    assert_close(u.float().cpu().numpy()[rows], ref, "pre-activation")
    assert_close(g.float().cpu().numpy()[rows], orc64.gelu(ref), "gelu")
    assert_close(r.float().cpu().numpy()[rows], ref + res[rows], "residual")


@pytest.mark.parametrize("M,kin,out", [(700, 256, 392), (300, 448, 392), (2144, 768, 768), (1000, 64, 3072), (333, 1536, 264),
                                       (257, 128, 8), (65, 192, 576)])
def test_every_tile_shape_gives_the_same_bits(env, orc64, M, kin, out):
    """Both kernel families, every block-tile shape, every epilogue form (bias; GELU with the stored pre-activation;
    residual; GELU' of a stored tensor in the input-gradient product of Eq. 2), on products whose rows and columns end
    inside a tile and whose contraction is 1 .. 24 k-tiles: the same bits as the default shape, which is checked
    against the oracle."""
    torch, P = env
    rng = np.random.default_rng(M * 3 + kin + out)
    x = bf16_np(rng, (M, kin)); w = bf16_np(rng, (kin, out), 0.05); b = rng.standard_normal(out).astype(np.float32)
    res = bf16_np(rng, (M, out)); aux = bf16_np(rng, (M, out))
    xt = to_dev(torch, x, torch.bfloat16)
    wt = to_dev(torch, np.ascontiguousarray(w.T), torch.bfloat16)
    bt = to_dev(torch, b); rt = to_dev(torch, res, torch.bfloat16); at = to_dev(torch, aux, torch.bfloat16)
    bits = lambda t: t.view(torch.int16).cpu().numpy().copy()

    def forms(tile):
        y, used = P.bsr_linear_forward(xt, wt, bt, tile=tile)
        u = torch.full((M, out), -7.0, dtype=torch.bfloat16, device="cuda")
        g, _ = P.bsr_linear_forward(xt, wt, bt, act=1, u_out=u, tile=tile)
        r, _ = P.bsr_linear_forward(xt, wt, bt, res=rt, tile=tile)
        # the same product seen as an input gradient: dy = x, W stored [in', out'] = w_t, times GELU'(aux)
        d, _ = P.bsr_linear_dgrad(xt, wt, u=at, tile=tile)
        torch.cuda.synchronize()
        assert used == 1
        return [bits(t) for t in (y, u, g, r, d)]

    base = forms(0)
    ref = orc64.linear(x, w, b)
    assert_close(torch.from_numpy(base[0]).view(torch.bfloat16).float().numpy(), ref, "linear")
    assert_close(torch.from_numpy(base[3]).view(torch.bfloat16).float().numpy(), ref + res, "residual")
    assert_close(torch.from_numpy(base[4]).view(torch.bfloat16).float().numpy(),
                 orc64.gelu_bwd(orc64.linear_dgrad(x, np.ascontiguousarray(w.T)), aux), "dgrad * GELU'")
    for tile in P.bsr_gemm_tile_shapes():
        for name, a, c in zip(("plain", "pre-activation", "gelu", "residual", "dgrad"), base, forms(tile)):
            assert np.array_equal(a, c), f"tile shape {tile}, {name}: {int(np.sum(a != c))} of {a.size} elements differ"
    with pytest.raises(P.BsrError):
        P.bsr_linear_forward(xt, wt, bt, tile=4242)


LN_SHAPES = [(6304, 768, 2304), (4416, 768, 3072), (2144, 768, 2304), (333, 128, 72), (1, 64, 8), (130, 768, 136)]


@pytest.mark.parametrize("M,kin,out", LN_SHAPES)
def test_layernorm_folded_into_linear(env, orc64, M, kin, out):
    """LayerNorm then linear (the LN -> qkv / LN -> fc1 pairs of the pre-norm block) as the frozen prefix runs
    them: one product on the raw rows with folded weights, statistics taken inside the kernel.  Against the
    oracle's LayerNorm followed by its linear layer on sampled rows; rows get different means and spreads."""
    torch, P = env
    rng = np.random.default_rng(11 * M + kin + out)
    x = S.round_to_bf16((rng.standard_normal((M, kin)) * rng.uniform(0.3, 3.0, (M, 1)) + rng.normal(0, 1.0, (M, 1))).astype(np.float32))
    w = (rng.standard_normal((kin, out)) * 0.05).astype(np.float32); b = rng.standard_normal(out).astype(np.float32)
    gamma = (1 + 0.2 * rng.standard_normal(kin)).astype(np.float32); beta = (0.1 * rng.standard_normal(kin)).astype(np.float32)
    rows = np.unique(np.concatenate([rng.choice(M, min(M, 192), replace=False), np.arange(max(0, M - 40), M)]))
    wf, cs, bf = P.bsr_ln_linear_fold(to_dev(torch, w), to_dev(torch, b), to_dev(torch, gamma), to_dev(torch, beta))
    xt = to_dev(torch, x, torch.bfloat16)
    y = P.bsr_ln_linear_forward(xt, wf, cs, bf, eps=1e-6)
    g = P.bsr_ln_linear_forward(xt, wf, cs, bf, eps=1e-6, act=1)
    torch.cuda.synchronize()
    ref = orc64.linear(orc64.layernorm(x[rows], gamma, beta, 1e-6)[0], w, b)
    assert_close(y.float().cpu().numpy()[rows], ref, "LayerNorm + linear")
    assert_close(g.float().cpu().numpy()[rows], orc64.gelu(ref), "LayerNorm + linear + GELU")
    # the folded tensors themselves: W' = diag(gamma) W rounded to bf16, its column sums, b' = b + beta W
    wp = S.round_to_bf16((w * gamma[:, None]).astype(np.float32))
    assert np.array_equal(wf.float().cpu().numpy(), wp.T)
    assert np.abs(cs.cpu().numpy() - wp.sum(0, dtype=np.float64)).max() <= 1e-5 * np.abs(wp).sum(0).max()
    assert np.abs(bf.cpu().numpy() - (b + beta.astype(np.float64) @ w)).max() <= 1e-5 * (np.abs(b).max() + 1)
    # every block-tile shape gives the same bits (the statistics are summed in an order of their own)
    y0 = y.view(torch.int16).cpu().numpy()
    for tile in P.bsr_gemm_tile_shapes():
        yt = P.bsr_ln_linear_forward(xt, wf, cs, bf, eps=1e-6, tile=tile)
        torch.cuda.synchronize()
        assert np.array_equal(yt.view(torch.int16).cpu().numpy(), y0), f"tile shape {tile} changes the result"


def test_layernorm_folded_refuses_what_it_cannot_take(env):
    torch, P = env
    x = torch.zeros((8, 96), dtype=torch.bfloat16, device="cuda")          # 96 is not a multiple of 64
    wf = torch.zeros((16, 96), dtype=torch.bfloat16, device="cuda"); v = torch.zeros(16, device="cuda")
    with pytest.raises(P.BsrError):
        P.bsr_ln_linear_forward(x, wf, v, v)
    x = torch.zeros((8, 64), dtype=torch.bfloat16, device="cuda"); wf = torch.zeros((16, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(P.BsrError):
        P.bsr_ln_linear_forward(x, wf, v, v, tile=12345)


@pytest.mark.parametrize("M,kin,out", SHAPES)
def test_linear_dgrad(env, orc64, M, kin, out):
    torch, P = env
    rng = np.random.default_rng(7 * M + kin + out)
    dy = bf16_np(rng, (M, out)); w = bf16_np(rng, (kin, out), 0.05); u = bf16_np(rng, (M, kin))
    rows = np.unique(np.concatenate([rng.choice(M, min(M, 192), replace=False), np.arange(max(0, M - 40), M)]))
    dyt = to_dev(torch, dy, torch.bfloat16); wst = to_dev(torch, w, torch.bfloat16)
    dx, used = P.bsr_linear_dgrad(dyt, wst)
    du, _ = P.bsr_linear_dgrad(dyt, wst, u=to_dev(torch, u, torch.bfloat16))
    torch.cuda.synchronize()
    assert used == 1
    ref = orc64.linear_dgrad(dy[rows], w)                       # Eq. 2
    assert_close(dx.float().cpu().numpy()[rows], ref, "dgrad")
    assert_close(du.float().cpu().numpy()[rows], orc64.gelu_bwd(ref, u[rows]), "dgrad * GELU'")


@pytest.mark.parametrize("M,kin,out", [(3072, 768, 2304), (2144, 3072, 768), (2144, 768, 3072),
                                       (3072, 768, 768), (333, 200, 72), (1, 64, 8), (67, 136, 776)])
def test_linear_wgrad(env, orc64, M, kin, out):
    torch, P = env
    rng = np.random.default_rng(3 * M + kin + out)
    x = bf16_np(rng, (M, kin)); dy = bf16_np(rng, (M, out))
    cols = np.unique(rng.choice(kin, min(kin, 96), replace=False))    # rows of dW are independent
    xt, dyt = to_dev(torch, x, torch.bfloat16), to_dev(torch, dy, torch.bfloat16)
    db = [torch.full((out,), float("nan"), dtype=torch.float32, device="cuda") for _ in range(3)]
    dw, used = P.bsr_linear_wgrad(xt, dyt, db=db[0])
    dw_nob, _ = P.bsr_linear_wgrad(xt, dyt)                             # db is optional
    ws = torch.empty(8 * (kin + 1) * out, dtype=torch.float32, device="cuda")
    dw_split, _ = P.bsr_linear_wgrad(xt, dyt, workspace=ws, db=db[1])  # split over the token sum
    dw_again, _ = P.bsr_linear_wgrad(xt, dyt, workspace=ws, db=db[2])
    torch.cuda.synchronize()
    assert used == 1, "the MFMA kernel must take this shape"
    ref, _ = orc64.linear_wgrad(np.ascontiguousarray(x[:, cols]), dy)  # Eq. 4
    _, ref_db = orc64.linear_wgrad(np.ascontiguousarray(x[:, :1]), dy)
    assert_close(dw.cpu().numpy()[cols], ref, "wgrad", tol=2e-3)
    assert torch.equal(dw, dw_nob)
    assert_close(dw_split.cpu().numpy()[cols], ref, "wgrad split-K", tol=2e-3)
    assert_close(db[0].cpu().numpy(), ref_db, "bias grad", tol=2e-3)
    assert_close(db[1].cpu().numpy(), ref_db, "bias grad split-K", tol=2e-3)
    assert torch.equal(dw_split, dw_again) and torch.equal(db[1], db[2]), "split-K must be bit-reproducible"


ATTN_SHAPES = [(2, 197, 12), (2, 138, 12), (3, 96, 6), (2, 67, 12), (2, 25, 3), (1, 1, 2), (2, 33, 2), (1, 256, 2)]


@pytest.mark.parametrize("B,T,H", ATTN_SHAPES)
def test_attention_forward(env, orc64, B, T, H):
    torch, P = env
    rng = np.random.default_rng(B * 1000 + T + H)
    qkv = bf16_np(rng, (B, T, 3 * H * 64), 1.5)          # logits with std ~ 2: a peaky softmax
    out, lse, cls, used = P.bsr_attention_forward(to_dev(torch, qkv, torch.bfloat16), H)
    torch.cuda.synchronize()
    assert used == 1, "the MFMA kernel must take head size 64 and T <= 256"
    Pm, o = orc64.attention(qkv, H)                       # Eq. 1
    assert_close(out.float().cpu().numpy(), o, "attention output")
    assert_close(cls.cpu().numpy(), Pm[:, :, 0, :], "CLS softmax row", tol=2e-3)   # fp32 by-product (Eq. 6)
    s = np.einsum("bihe,bjhe->bhij", qkv[..., :H * 64].reshape(B, T, H, 64).astype(np.float64),
                  qkv[..., H * 64:2 * H * 64].reshape(B, T, H, 64).astype(np.float64)) / 8.0
    ref_lse = np.log(np.exp(s - s.max(-1, keepdims=True)).sum(-1)) + s.max(-1)
    assert np.max(np.abs(lse.cpu().numpy() - ref_lse)) < 1e-3
    assert abs(float(cls.sum(-1).mean().item()) - 1.0) < 1e-5      # softmax rows sum to 1


@pytest.mark.parametrize("B,T,H", ATTN_SHAPES)
def test_attention_backward(env, orc64, B, T, H):
    torch, P = env
    rng = np.random.default_rng(B * 999 + T + H)
    qkv = bf16_np(rng, (B, T, 3 * H * 64), 1.0)
    dout = bf16_np(rng, (B, T, H * 64), 1.0)
    qt = to_dev(torch, qkv, torch.bfloat16)
    out, lse, _, _ = P.bsr_attention_forward(qt, H)
    dqkv, used = P.bsr_attention_backward(qt, out, to_dev(torch, dout, torch.bfloat16), lse, H)
    torch.cuda.synchronize()
    assert used == 1
    Pm, _ = orc64.attention(qkv, H)
    ref = orc64.attention_bwd(qkv, Pm, dout, H)           # Eq. 3, 5
    got = dqkv.float().cpu().numpy()
    D = H * 64
    for name, sl in (("dq", slice(0, D)), ("dk", slice(D, 2 * D)), ("dv", slice(2 * D, 3 * D))):
        assert_close(got[..., sl], ref[..., sl], name, tol=1.5e-2)
