"""GPU parity at the edges of the method: drop locations that keep nothing or everything, one image,
the deepest model the library takes, and what the entry points refuse."""
import numpy as np
import pytest

import bsr_synth as S
from test_gpu_parity import TOL_BF16, TOL_FP32, check_step, hip  # noqa: F401  (hip is a fixture)

pytestmark = pytest.mark.gpu

EDGES = [
    ("keep_nothing", dict(keep_ratio=0.001)),            # K = floor(r n) = 0: only the class token survives
    ("keep_everything", dict(keep_k=[64, 64])),         # a drop location that drops nothing
    ("keep_then_nothing", dict(keep_k=[64, 0])),
    ("one_image", dict(batch=1)),
    ("deepest", dict(depth=16, first_trainable=13, drop_blocks=[2, 9, 15], keep_k=[40, 17, 5])),
    ("all_trainable_drop_in_block_0", dict(first_trainable=0, drop_blocks=[0], keep_k=[33])),
]


@pytest.mark.parametrize("dtype,tol", [("fp32", TOL_FP32), ("bf16", TOL_BF16)])
@pytest.mark.parametrize("label,over", EDGES, ids=[e[0] for e in EDGES])
def test_edge_configurations_match_the_oracle(hip, orc64, label, over, dtype, tol):
    cfg = S.get_config("mini_4blk", dtype=dtype, **over)
    p = S.make_params(cfg, std=0.05)
    x, y = S.make_inputs(cfg)
    got, ref, _ = check_step(hip, orc64, cfg, p, x, y, tol, free_running=False)
    for i, k in enumerate(ref["keep_k"]):
        assert got["kept_idx"][i].shape == (x.shape[0], k)


def test_fused_token_when_nothing_or_everything_is_dropped(hip, orc64):
    # nothing kept: the fused token is the importance-weighted mean of all patch tokens;
    # everything kept: there is nothing to fuse and no token is appended
    for over in (dict(keep_ratio=0.001), dict(keep_k=[64, 64])):
        cfg = S.get_config("mini_4blk", dtype="fp32", fuse_dropped=True, **over)
        p = S.make_params(cfg, std=0.05)
        x, y = S.make_inputs(cfg)
        check_step(hip, orc64, cfg, p, x, y, TOL_FP32, free_running=False)


def test_entry_points_refuse_bad_arguments(hip):
    import torch
    import paper_2405_10951_amd as P
    cfg = S.get_config("mini_4blk", dtype="bf16")
    p = S.make_params(cfg)
    ctx = P.Context(cfg, p, 4)
    dev = torch.device("cuda:0")
    x, _ = S.make_inputs(cfg)
    xin = torch.as_tensor(x).to(dev).to(ctx.act_dtype).contiguous()       # batch 5 > max_batch 4
    with pytest.raises(P.BsrError):
        ctx.bsr_forward_frozen(xin)
    ok = ctx.bsr_forward_frozen(xin[:4].contiguous())
    with pytest.raises(P.BsrError):                                          # misaligned input pointer
        ctx.bsr_forward_frozen(xin.view(-1)[1:1 + 4 * xin[0].numel()].view(4, *xin.shape[1:]))
    lab = torch.zeros(4, dtype=torch.int32, device=dev)
    with pytest.raises(P.BsrError):                                          # gradients missing
        ctx._chk(ctx.lib.bsr_train_blocks_fwd_bwd(ctx.ctx, ok.data_ptr(), lab.data_ptr(), 4,
                                                  torch.zeros(1, device=dev).data_ptr(), None, None, None,
                                                  None, None, None, None))
    torch.cuda.synchronize()


def test_selection_with_nan_scores_keeps_exactly_k(hip, orc32):
    """A NaN score (a diverged step) ranks last, like minus infinity: exactly K indices come out, ascending, all
    valid, equal to the reference ranking of the scores with NaN replaced by -inf.  The slots behind the K-th and
    the neighbouring images' slots stay untouched."""
    import torch
    import paper_2405_10951_amd as P
    cfg = S.get_config("mini_4blk", dtype="bf16")
    ctx = P.Context(cfg, S.make_params(cfg), 4)
    rng = np.random.default_rng(5)
    for n, k in [(196, 137), (64, 44), (300, 7), (33, 33)]:
        B = 4
        a = rng.standard_normal((B, n)).astype(np.float32)
        a[0, ::3] = np.nan                       # a third of the scores
        a[1, :] = np.nan                         # all of them: the first K indices
        a[2, n // 2] = np.nan
        x = rng.standard_normal((B, n + 1, cfg["dim"])).astype(np.float32)
        xt = torch.as_tensor(x).cuda().to(torch.bfloat16)
        guard = torch.full((B * k + 64,), -7, dtype=torch.int32, device="cuda")
        idx, _ = ctx.bsr_select_tokens(torch.as_tensor(a).cuda(), xt, k, idx_out=guard[:B * k].view(B, k))
        torch.cuda.synchronize()
        assert (guard[B * k:] == -7).all(), "wrote past the K-th slot of the last image"
        idx = idx.cpu().numpy()
        for b in range(B):
            ref = orc32.topk(np.where(np.isnan(a[b]), -np.inf, a[b]).astype(np.float32), k)
            assert np.array_equal(idx[b], ref), (n, k, b)
