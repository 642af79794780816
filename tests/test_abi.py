"""CPU-only checks of the C ABI: the built library loads, exports every function include/bsr.h
declares, and its host-only entry points (token schedule, workspace size, configuration checks)
behave as documented.  Nothing here launches a kernel."""
import ctypes as C
import os
import re

import pytest

import bsr_synth as S
import paper_2405_10951_amd as P
from oracle import token_schedule

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "bsr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bsr_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = P.load_library()
    names = declared_functions()
    assert {"bsr_init", "bsr_forward_frozen", "bsr_select_tokens", "bsr_train_blocks_fwd_bwd",
            "bsr_sgd_step"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/bsr.h but not exported"


def test_python_binding_has_the_entry_points_names():
    for n in ("bsr_forward_frozen", "bsr_select_tokens", "bsr_train_blocks_fwd_bwd", "bsr_sgd_step",
              "bsr_refresh_weights", "bsr_profile_begin", "bsr_profile_end", "bsr_destroy"):
        assert hasattr(P.Context, n)
    for n in ("bsr_token_schedule", "bsr_workspace_bytes", "bsr_linear_forward", "bsr_linear_dgrad",
              "bsr_linear_wgrad", "bsr_attention_forward", "bsr_attention_backward"):
        assert hasattr(P, n)


@pytest.mark.parametrize("name,keep,expect", [("c3_vit_b", 0.7, [137, 95, 66]), ("c3_vit_b", 0.5, [98, 49, 24]),
                                              ("c3_vit_b", 1.0, [196, 196, 196]), ("c1_block_fp32", 0.7, [44])])
def test_token_schedule_matches_the_paper_and_the_oracle(name, keep, expect):
    cfg = S.get_config(name, keep_ratio=keep)
    kk, ta, tm = P.bsr_token_schedule(P.make_config(cfg, 4))
    assert kk == expect                                   # N/2, N/4, N/8 at drop rate 0.5 (Sec. 4.3)
    n0 = S.tokens_at_input(cfg) - 1
    assert kk == token_schedule(n0, keep, len(cfg["drop_blocks"]))
    for i, blk in enumerate(cfg["drop_blocks"]):
        assert tm[blk] == kk[i] + 1 and ta[blk] == (n0 + 1 if i == 0 else kk[i - 1] + 1)


def test_explicit_keep_k_wins_over_the_ratio():
    cfg = S.get_config("c2_deit_s", keep_k=[12, 8, 4])
    kk, _, tm = P.bsr_token_schedule(P.make_config(cfg, 2))
    assert kk == [12, 8, 4] and tm[-1] == 5


def test_workspace_grows_with_batch_and_trainable_blocks():
    cfg = S.get_config("c3_vit_b")
    a = P.bsr_workspace_bytes(P.make_config(cfg, 32))
    b = P.bsr_workspace_bytes(P.make_config(cfg, 64))
    c = P.bsr_workspace_bytes(P.make_config(dict(cfg, first_trainable=0), 32))
    assert 0 < a < b and a < c


@pytest.mark.parametrize("bad", [dict(dim=770), dict(heads=5), dict(depth=17), dict(drop_blocks=[6, 3, 9]),
                                 dict(drop_blocks=[3, 6, 12]), dict(keep_ratio=0.0), dict(keep_ratio=1.5),
                                 dict(first_trainable=13), dict(loss=S.LOSS_MEAN_SQ), dict(num_classes=0),
                                 dict(image_size=225), dict(keep_k=[300, 10, 5]), dict(mlp_hidden=3071)])
def test_bad_configurations_are_rejected_with_a_message(bad):
    cfg = S.get_config("c3_vit_b", **bad)
    with pytest.raises(P.BsrError) as e:
        P.bsr_workspace_bytes(P.make_config(cfg, 8))
    assert e.value.code == -2 and len(str(e.value)) > 20


def test_max_batch_must_be_positive_and_null_arguments_fail():
    cfg = S.get_config("c3_vit_b")
    with pytest.raises(P.BsrError):
        P.bsr_workspace_bytes(P.make_config(cfg, 0))
    lib = P.load_library()
    assert lib.bsr_workspace_bytes(None, None) == -1
    assert lib.bsr_token_schedule(None, None, None, None) == -1
    assert lib.bsr_destroy(None) == 0
    assert lib.bsr_last_error(None) is not None


def test_step_flop_count_matches_the_closed_form():
    # product-side counter used by the benchmark against the oracle-side MAC count (Table 4's 2249 GMacs)
    from paper_2405_10951_amd.flops import step_flops
    from oracle import accounting as acc
    tb = acc.tokens_per_block(197, 12, [], [])
    macs = acc.forward_macs(tb, 768, 3072, 196, 768, 100)
    fl = step_flops(768, 3072, 100, 768, 196, [197] * 12, [197] * 12, 12, 1)
    assert abs((fl["fwd_gemm"] + fl["fwd_attn"] + fl["head"] / 3) / (2 * macs) - 1) < 1e-9
    c3 = step_flops(768, 3072, 100, 768, 196, [197, 197, 197, 197, 138, 138, 138, 96, 96, 96, 67, 67],
                    [197, 197, 197, 138, 138, 138, 96, 96, 96, 67, 67, 67], 8, 32)
    assert abs(c3["total"] / 1e9 - 1012.8) < 0.5
