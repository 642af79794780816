"""The allocation-free weight-gradient entry point (split-K scratch in an array that is part of the library)
against the entry point that takes its scratch from the caller: same kernels, same split, so the same bits; and
against the oracle's Eq. 4 at the tolerance of the kernel-level tests.  Two calls in a row, the second on a
smaller layer, so that what the first left in the shared array is there when the second runs."""
import numpy as np
import pytest

import bsr_synth as S

pytestmark = pytest.mark.gpu

SCRATCH_FLOATS = 6 << 20          # the size the header states


def _case(torch, P, orc64, M, kin, out, seed):
    rng = np.random.default_rng(seed)
    x = S.round_to_bf16(rng.standard_normal((M, kin)).astype(np.float32))
    dy = S.round_to_bf16((rng.standard_normal((M, out)) * 0.1).astype(np.float32))
    xt = torch.as_tensor(x).cuda().to(torch.bfloat16)
    dyt = torch.as_tensor(dy).cuda().to(torch.bfloat16)
    # reference entry point, with a caller workspace of the same size as the built-in array (same split-K plan)
    ws = torch.empty(SCRATCH_FLOATS, dtype=torch.float32, device="cuda")
    dw_ref = torch.full((kin, out), float("nan"), dtype=torch.float32, device="cuda")
    db_ref = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda")
    _, used_ref = P.bsr_linear_wgrad(xt, dyt, dw=dw_ref, workspace=ws, db=db_ref)
    dw = torch.full((kin, out), float("nan"), dtype=torch.float32, device="cuda")
    db = torch.full((out,), float("nan"), dtype=torch.float32, device="cuda")
    _, used = P.bsr_linear_wgrad_static(xt, dyt, dw=dw, db=db)
    torch.cuda.synchronize()
    assert used == used_ref == 1
    assert torch.equal(dw, dw_ref), f"dw differs from bsr_linear_wgrad at M={M} in={kin} out={out}"
    assert torch.equal(db, db_ref), f"db differs from bsr_linear_wgrad at M={M} in={kin} out={out}"
    ref_w, ref_b = orc64.linear_wgrad(x, dy)
    got_w, got_b = dw.cpu().numpy().astype(np.float64), db.cpu().numpy().astype(np.float64)
    assert np.abs(got_w - ref_w).max() <= 2e-3 * np.abs(ref_w).max()
    assert np.abs(got_b - ref_b).max() <= 2e-3 * np.abs(ref_b).max()


def test_static_scratch_weight_gradient_twice(orc64):
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device")
    import paper_2405_10951_amd as P
    _case(torch, P, orc64, 3072, 768, 3072, 1)      # fc1 of ViT-B at the trained blocks' token count: split-K
    _case(torch, P, orc64, 1100, 384, 1152, 2)      # a smaller layer right after it, ragged token count


def test_static_scratch_refuses_a_layer_beyond_its_limit():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device")
    import paper_2405_10951_amd as P
    x = torch.zeros((64, 2048), dtype=torch.bfloat16, device="cuda")
    dy = torch.zeros((64, 2048), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(P.BsrError) as e:
        P.bsr_linear_wgrad_static(x, dy)          # 2 * 2049 * 2048 floats > 6 Mi
    assert "scratch" in str(e.value)
