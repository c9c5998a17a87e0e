"""Kernel timing spans of the library (benchmark aid): selection of kinds."""
import pytest
import torch

from paper_2604_02715_amd import binding as B
from paper_2604_02715_amd import inputs

pytestmark = pytest.mark.gpu


def test_profile_brackets_only_the_selected_kinds():
    from gpu_common import build_pool
    cfg = inputs.CONFIGS["c1_tiny"]
    pool, dense = build_pool(cfg, seed=0)
    try:
        x = inputs.activations(cfg, 0, seed=0).cuda()
        ids, g = inputs.routing(cfg, 0, seed=0)
        idd, gd = torch.from_numpy(ids).cuda(), torch.from_numpy(g).cuda()
        out = torch.zeros((cfg.tokens, cfg.hidden), dtype=torch.float32, device="cuda")
        union = inputs.routed_union(ids)
        pool.reset_page_table()

        def step():
            pool.materialize(0, union, list(range(len(union))))
            pool.expert_ffn(0, x, idd, gd, out)

        B.fluxmoe_profile_enable(pool.ctx, True)
        B.fluxmoe_profile_collect(pool.ctx)
        step(); step()
        prof = B.fluxmoe_profile_collect(pool.ctx)
        assert all(prof[k][1] == 2 and prof[k][0] > 0 for k in B.PROFILE_KINDS)

        B.fluxmoe_profile_enable(pool.ctx, True, only_kinds=("decode",))
        step(); step(); step()
        prof = B.fluxmoe_profile_collect(pool.ctx)
        assert prof["decode"][1] == 3 and prof["decode"][0] > 0
        assert all(prof[k] == (0.0, 0) for k in B.PROFILE_KINDS if k != "decode")

        B.fluxmoe_profile_enable(pool.ctx, True, only_kinds=("gemm1_swiglu", "combine"))
        step()
        prof = B.fluxmoe_profile_collect(pool.ctx)
        assert [prof[k][1] for k in B.PROFILE_KINDS] == [0, 0, 1, 0, 1]

        B.fluxmoe_profile_enable(pool.ctx, False)
        step()
        assert all(v == (0.0, 0) for v in B.fluxmoe_profile_collect(pool.ctx).values())
        torch.cuda.synchronize()
        assert pool.device_errors() == 0
    finally:
        pool.close()
