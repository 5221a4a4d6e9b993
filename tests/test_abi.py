"""The C-ABI library: every declared symbol is exported, and host-side
validation returns the documented status codes (no GPU needed: validation
runs before any launch)."""
import ctypes
import os
import re

import pytest

import paper_2601_08800_amd as moe
from paper_2601_08800_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def cfg(**kw):
    base = dict(hidden=256, n_experts=8, top_k=2, score_fn=0, renormalize=1, routed_scale=1.0,
                n_groups=1, topk_groups=1, group_score_n=0, expert_lo=0, expert_hi=8,
                inter_local=512, act_dtype=B.MOE_BF16, weight_dtype=B.MOE_BF16)
    base.update(kw)
    return moe.MoEConfig(**base)


def test_header_symbols_are_exported():
    hdr = open(os.path.join(ROOT, "include", "moe.h")).read()
    declared = set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    lib = ctypes.CDLL(moe.lib_path())
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_mirror_matches_header():
    hdr = open(os.path.join(ROOT, "include", "moe.h")).read()
    body = hdr[hdr.index("typedef struct {"):hdr.index("} moe_config;")]
    fields = re.findall(r"^\s*(?:int32_t|float)\s+(\w+);", body, re.M)
    assert fields == [f[0] for f in moe.MoEConfig._fields_]
    assert ctypes.sizeof(moe.MoEConfig) == 4 * len(fields)


def test_workspace_bytes():
    assert moe.moe_workspace_bytes(cfg(), 0) > 0
    assert moe.moe_workspace_bytes(cfg(), 64) >= 64 * 8 * 4
    assert moe.moe_workspace_bytes(cfg(top_k=9), 64) == 0       # invalid config
    assert moe.moe_workspace_bytes(cfg(), -1) == 0


def status_of(fn, *a):
    try:
        fn(*a)
    except moe.MoEError as e:
        return e.status
    return B.MOE_OK


P = 0x1000      # any aligned non-NULL value: validation fails before it is dereferenced


@pytest.mark.parametrize("kw", [dict(hidden=0), dict(hidden=100), dict(top_k=0), dict(top_k=9),
                                dict(n_groups=3), dict(n_groups=4, topk_groups=5, group_score_n=1),
                                dict(n_groups=4, topk_groups=2, group_score_n=3),
                                dict(n_groups=4, topk_groups=1, group_score_n=1, top_k=3),
                                dict(expert_lo=4, expert_hi=4), dict(expert_hi=9),
                                dict(inter_local=12), dict(score_fn=2),
                                dict(routed_scale=float("nan"))])
def test_invalid_configs(kw):
    c = cfg(**kw)
    assert status_of(moe.moe_route, c, 4, P, P, None, None, None, P, P, P, None, 1 << 30) == B.MOE_ERR_INVALID_ARG
    assert status_of(moe.moe_combine, c, 4, P, P, P, None, P) == B.MOE_ERR_INVALID_ARG


@pytest.mark.parametrize("kw", [dict(act_dtype=B.MOE_F32), dict(act_dtype=3),
                                dict(weight_dtype=B.MOE_FP8_E4M3_B128, inter_local=192),
                                dict(n_experts=1024, expert_hi=8), dict(top_k=33, n_experts=64)])
def test_unsupported(kw):
    c = cfg(**kw)
    assert status_of(moe.moe_dispatch, c, 4, P, P, P, P, P, P, P, P, None, 1 << 30) == B.MOE_ERR_UNSUPPORTED


def test_pointer_and_size_checks():
    c = cfg()
    big = 1 << 30
    assert status_of(moe.moe_route, c, -1, P, P, None, None, None, P, P, P, None, big) == B.MOE_ERR_INVALID_ARG
    assert status_of(moe.moe_route, c, 4, None, P, None, None, None, P, P, P, None, big) == B.MOE_ERR_INVALID_ARG
    assert status_of(moe.moe_route, c, 4, P + 4, P, None, None, None, P, P, P, None, big) == B.MOE_ERR_INVALID_ARG
    assert status_of(moe.moe_route, c, 4, P, P, None, None, None, P, P, P, None, 16) == B.MOE_ERR_WORKSPACE
    assert status_of(moe.moe_dispatch, c, 4, P, P, P, P, P, P, P, P, None, 0) == B.MOE_ERR_WORKSPACE
    assert status_of(moe.moe_dispatch, c, 4, P, P, P, None, P, P, P, P, None, big) == B.MOE_ERR_INVALID_ARG
    assert status_of(moe.moe_expert_ffn, c, 0, P, P, 8, P, P, P, None, None, None, P, P, None, big) == B.MOE_ERR_INVALID_ARG
    assert status_of(moe.moe_expert_ffn, c, 8, P, P, 8, P, P, P, None, None, None, P, P, None, 8) == B.MOE_ERR_WORKSPACE
    f8 = cfg(weight_dtype=B.MOE_FP8_E4M3_B128)
    assert status_of(moe.moe_expert_ffn, f8, 8, P, P, 8, P, P, P, None, None, None, P, P, None, big) == B.MOE_ERR_INVALID_ARG
    assert status_of(moe.moe_combine, c, 4, P, None, P, None, P) == B.MOE_ERR_INVALID_ARG
    # T == 0 and zero capacity are no-ops
    assert status_of(moe.moe_route, c, 0, None, None, None, None, None, None, None, None, None, 0) == B.MOE_OK
    assert status_of(moe.moe_dispatch, c, 0, None, None, None, None, None, None, None, None, None, 0) == B.MOE_OK
    assert status_of(moe.moe_expert_ffn, c, 8, None, None, 0, None, None, None, None, None, None, None, None, None, 0) == B.MOE_OK
    assert status_of(moe.moe_combine, c, 0, None, None, None, None, None) == B.MOE_OK
    assert moe.moe_status_string(B.MOE_ERR_WORKSPACE) == "workspace too small"


def test_shard_arguments_are_validated():
    c = cfg()
    args = lambda r, m: (c, 8, P, P, r, m, P, P, P, P, P, P, None, 1 << 30)
    bad = [(-1, 2), (2, 2), (0, 0), (0, 3), (0, 64)]     # rank out of range; H=256 not divisible / shard not whole pieces
    for r, m in bad:
        assert status_of(moe.moe_dispatch_shard, *args(r, m)) == B.MOE_ERR_INVALID_ARG
    assert status_of(moe.moe_combine_stage, c, 8, P, P, P, 3, 0, P) == B.MOE_ERR_INVALID_ARG
    assert status_of(moe.moe_combine_stage, c, 8, P, P, P, 2, 2, P) == B.MOE_ERR_INVALID_ARG
    assert status_of(moe.moe_combine_stage, c, 8, None, P, P, 2, 0, P) == B.MOE_ERR_INVALID_ARG
    assert status_of(moe.moe_combine_stage, c, 0, None, None, None, 2, 0, None) == B.MOE_OK
