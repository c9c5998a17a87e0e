"""fluxmoe_expert_ffn_static (the entry point that allocates nothing: FFN scratch in a static device
array) against fluxmoe_expert_ffn (scratch in the bound workspace) through the C ABI: two calls in a
row, the second with a smaller batch, both bit-equal to the existing entry point's output (the kernels
are deterministic) and within 1e-3 relative Frobenius error of the FP64 oracle; a batch whose scratch
exceeds the static array is refused with ENOMEM and enqueues nothing."""
import numpy as np
import pytest
import torch

from oracle import ffn as offn
from paper_2604_02715_amd import binding as B
from paper_2604_02715_amd import harness, inputs

pytestmark = pytest.mark.gpu
TOL = 1e-3


def test_static_scratch_ffn_matches_workspace_ffn_twice():
    cfg = inputs.CONFIGS["c1_tiny"]
    pool = harness.ExpertPool(cfg)
    try:
        w13, w2 = harness.make_layer_on_host(cfg)
        pool.bind_layer(0, pool.encode_layer(0, w13, w2))
        pool.reset_page_table()
        slots = inputs.slot_permutation(cfg.n_slots, "no_alloc")
        pool.materialize(0, np.arange(cfg.n_experts), slots)
        torch.cuda.synchronize()
        x_all = inputs.activations(cfg)
        ids_all, g_all = inputs.routing(cfg)
        weights = lambda e: (inputs.bits_u16(w13[e]), inputs.bits_u16(w2[e]))
        sptr = torch.cuda.current_stream().cuda_stream
        for T in (cfg.tokens, 24):                      # the second call is smaller and sees the first call's leftovers
            assert B.fluxmoe_ffn_workspace_bytes(pool.ctx, T, cfg.top_k) <= B.STATIC_SCRATCH_BYTES
            x = x_all[:T].contiguous().cuda()
            ids = torch.from_numpy(ids_all[:T].copy()).cuda()
            g = torch.from_numpy(g_all[:T].copy()).cuda()
            ref = torch.full((T, cfg.hidden), 7.0, dtype=torch.float32, device="cuda")
            got = torch.full((T, cfg.hidden), -7.0, dtype=torch.float32, device="cuda")
            pool.expert_ffn(0, x, ids, g, ref)
            B.fluxmoe_expert_ffn_static(pool.ctx, 0, x.data_ptr(), T, ids.data_ptr(), g.data_ptr(), cfg.top_k,
                                        pool.page_table.data_ptr(), got.data_ptr(), 0, sptr)
            torch.cuda.synchronize()
            assert pool.device_errors() == 0
            assert torch.equal(got, ref), "static-scratch FFN differs from the workspace FFN at T=%d" % T
            want = offn.moe_ffn(inputs.bits_u16(x_all[:T].contiguous()), ids_all[:T], g_all[:T], weights, round_h=True)
            err = offn.rel_frobenius(got.cpu().numpy(), want)
            print("T=%d rel. Frobenius error vs oracle %.3e" % (T, err), flush=True)
            assert err <= TOL
        # too large for the static array: refused before anything is enqueued
        T_big = 16384
        assert B.fluxmoe_ffn_workspace_bytes(pool.ctx, T_big, cfg.top_k) > B.STATIC_SCRATCH_BYTES
        x = torch.zeros((T_big, cfg.hidden), dtype=torch.bfloat16, device="cuda")
        ids = torch.zeros((T_big, cfg.top_k), dtype=torch.int32, device="cuda")
        g = torch.zeros((T_big, cfg.top_k), dtype=torch.float32, device="cuda")
        out = torch.full((T_big, cfg.hidden), 5.0, dtype=torch.float32, device="cuda")
        with pytest.raises(B.FluxmoeError) as ei:
            B.fluxmoe_expert_ffn_static(pool.ctx, 0, x.data_ptr(), T_big, ids.data_ptr(), g.data_ptr(), cfg.top_k,
                                        pool.page_table.data_ptr(), out.data_ptr(), 0, sptr)
        assert ei.value.status == -2
        torch.cuda.synchronize()
        assert bool((out == 5.0).all())
    finally:
        pool.close()
