"""Two tiers, three streams, two slot halves (Sec. 3 sliding window, Sec. 4.2 host tier,
Alg. 1): results must equal the oracle layer by layer, and the overlapped schedule must give
exactly the bytes of the one-stream schedule."""
import numpy as np
import pytest
import torch

from oracle import ffn as offn
from paper_2604_02715_amd import binding as B
from paper_2604_02715_amd import harness, inputs

pytestmark = pytest.mark.gpu


def small_stream_cfg(**kw):
    base = dict(n_experts=12, hidden=256, ffn=384, tokens=48, top_k=4, n_slots=8, n_layers=5,
                host_fraction=0.40)
    base.update(kw)
    return inputs.scaled(inputs.CONFIGS["c5_stream"], **base)


def build(cfg):
    pool = harness.ExpertPool(cfg)
    dense, stats = {}, []
    for layer in range(cfg.n_layers):
        w13, w2 = harness.make_layer_on_host(cfg, layer)
        blob = pool.encode_layer(layer, w13, w2)
        stats.append(pool.bind_layer(layer, blob, cfg.host_fraction))
        dense[layer] = (w13, w2)
    max_host = max(s[1] for s in stats)
    pool.bind_staging(2 * max_host * 4096 + 8192)
    return pool, dense, stats


def test_host_tier_blocks_decode_like_hbm_blocks():
    cfg = small_stream_cfg(n_layers=2)
    pool, dense, stats = build(cfg)
    try:
        assert all(n_host == int(np.ceil(0.4 * n - 1e-12)) and n_host > 0 for n, n_host in stats)
        pool.poison_slots()
        pool.reset_page_table()
        # without a prefetch: materialize stages the blocks itself
        pool.materialize(0, [0, 5, 11, 3], [0, 1, 2, 3])
        # with a prefetch on a side stream for a superset, then two waves over subsets
        side = torch.cuda.Stream()
        pool.prefetch_host(1, list(range(12)), side)
        pool.materialize(1, [0, 1, 2, 3], [4, 5, 6, 7])
        torch.cuda.synchronize()
        assert pool.device_errors() == 0
        from gpu_common import assert_slot_equals
        for e, s in zip([0, 5, 11, 3], [0, 1, 2, 3]):
            assert_slot_equals(pool, s, dense[0][0][e], dense[0][1][e])
        for e, s in zip([0, 1, 2, 3], [4, 5, 6, 7]):
            assert_slot_equals(pool, s, dense[1][0][e], dense[1][1][e])
        pool.materialize(1, [8, 9, 10, 11], [4, 5, 6, 7])       # second wave, same staging half
        torch.cuda.synchronize()
        for e, s in zip([8, 9, 10, 11], [4, 5, 6, 7]):
            assert_slot_equals(pool, s, dense[1][0][e], dense[1][1][e])
    finally:
        pool.close()


def test_staging_too_small_is_an_error():
    cfg = small_stream_cfg(n_layers=1)
    pool, dense, stats = build(cfg)
    try:
        pool.bind_staging(2 * 4096)
        pool.reset_page_table()
        with pytest.raises(B.FluxmoeError) as ei:
            pool.materialize(0, [0, 1], [0, 1])
        assert ei.value.status == -2
    finally:
        pool.close()


def build_whole_tensor_tiers(cfg):
    """Every layer keeps three down tensors and one fused tensor dense in pinned host memory (tier 2),
    two more down tensors compressed in pinned host memory (tier 1), the rest compressed on the device."""
    pool = harness.ExpertPool(cfg)
    dense = {}
    E = cfg.n_experts
    for layer in range(cfg.n_layers):
        w13, w2 = harness.make_layer_on_host(cfg, layer)
        blob = pool.encode_layer(layer, w13, w2)
        pool.bind_layer(layer, blob, 0.0)
        pool.place_tensors_raw_on_host(layer, [((2, e), w2[e]) for e in (E - 1, E - 2, E - 3)] + [((1, E - 1), w13[E - 1])])
        pool.place_tensors_on_host(layer, blob, [(2, 0), (2, 1)])
        dense[layer] = (w13, w2)
    pool.bind_staging(2 * (3 * cfg.sigma2 + cfg.sigma1 + 2 * cfg.sigma2) + 16384)
    return pool, dense, None


@pytest.mark.parametrize("tiers", ["block_prefix", "whole_tensors_dense_and_compressed"])
def test_overlapped_schedule_matches_oracle_and_single_stream_schedule(tiers):
    cfg = small_stream_cfg(host_fraction=0.40 if tiers == "block_prefix" else 0.0)
    pool, dense, stats = build(cfg) if tiers == "block_prefix" else build_whole_tensor_tiers(cfg)
    try:
        routings = [inputs.routing(cfg, layer) for layer in range(cfg.n_layers)]
        xs_host = [inputs.activations(cfg, layer) for layer in range(cfg.n_layers)]
        xs = [x.cuda() for x in xs_host]
        outs = [torch.zeros((cfg.tokens, cfg.hidden), dtype=torch.float32, device="cuda")
                for _ in range(cfg.n_layers)]
        proxy = harness.StreamingProxy(pool, routings, xs, outs)
        assert max(len(w) for _, waves in proxy.plan for w, _ in waves) <= cfg.n_slots // 2
        assert any(len(waves) > 1 for _, waves in proxy.plan)          # waves are exercised
        pool.reset_page_table()
        torch.cuda.synchronize()
        results = []
        # one stream; overlapped; overlapped with every FFN held back ~0.2 ms (a missing
        # write-after-read wait would let the next materialize overwrite unread slots)
        for mode, delay in ((True, 0), (False, 0), (False, 400000)):
            for o in outs:
                o.fill_(float("nan"))
            pool.poison_slots()
            torch.cuda.synchronize()
            proxy.run_pass(single_stream=mode, ffn_delay_cycles=delay)
            torch.cuda.synchronize()
            assert pool.device_errors() == 0
            results.append([o.cpu().numpy().copy() for o in outs])
        for layer in range(cfg.n_layers):
            w13, w2 = dense[layer]
            want = offn.moe_ffn(inputs.bits_u16(xs_host[layer]), routings[layer][0], routings[layer][1],
                                lambda e: (inputs.bits_u16(w13[e]), inputs.bits_u16(w2[e])), round_h=True)
            err = offn.rel_frobenius(results[0][layer], want)
            print("layer", layer, "rel. Frobenius error %.3e" % err, flush=True)
            assert err <= 1e-3
            assert np.array_equal(results[0][layer], results[1][layer]), "overlap changed layer %d" % layer
            assert np.array_equal(results[0][layer], results[2][layer])
        assert (pool.page_table.cpu().numpy() == -1).all()             # everything was released
    finally:
        pool.close()


def test_single_layer_waves_with_release_on_another_stream():
    """One layer, two streams, repeated passes: every wave's release runs on the inference stream
    while the next wave's materialize (same layer, same page-table row, same slots) runs on the
    load stream.  The release must wait for the wave's FFN and the next materialize for the
    release, otherwise the table ends at -1 for mapped experts and the FFN silently drops them
    (Alg. 1's ordering applied to the page-table row)."""
    cfg = small_stream_cfg(n_layers=1, n_experts=12, n_slots=8, host_fraction=0.0)
    pool = harness.ExpertPool(cfg)
    try:
        w13, w2 = harness.make_layer_on_host(cfg, 0)
        pool.bind_layer(0, pool.encode_layer(0, w13, w2))
        routings = [inputs.routing(cfg, 0)]
        x_host = inputs.activations(cfg, 0)
        outs = [torch.zeros((cfg.tokens, cfg.hidden), dtype=torch.float32, device="cuda")]
        proxy = harness.StreamingProxy(pool, routings, [x_host.cuda()], outs)
        assert len(proxy.plan[0][1]) >= 2                               # several waves through 4 slots
        want = offn.moe_ffn(inputs.bits_u16(x_host), routings[0][0], routings[0][1],
                            lambda e: (inputs.bits_u16(w13[e]), inputs.bits_u16(w2[e])), round_h=True)
        pool.reset_page_table()
        torch.cuda.synchronize()
        first = None
        for rep, delay in enumerate((0, 300000, 0, 300000)):
            outs[0].fill_(float("nan"))
            torch.cuda.synchronize()
            proxy.run_pass(ffn_delay_cycles=delay)
            proxy.run_pass(ffn_delay_cycles=delay)                      # back to back: pass 2 reuses pass 1's slots
            torch.cuda.synchronize()
            assert pool.device_errors() == 0
            got = outs[0].cpu().numpy()
            err = offn.rel_frobenius(got, want)
            print("rep", rep, "rel. Frobenius error %.3e" % err, flush=True)
            assert err <= 1e-3
            if first is None:
                first = got.copy()
            assert np.array_equal(got, first)
            assert (pool.page_table.cpu().numpy() == -1).all()
    finally:
        pool.close()


def test_prefetch_of_some_experts_then_materialize_of_others_restages_in_order():
    """A fetch of experts A on a side stream, then a materialize of experts outside A on another
    stream: the materialize stages its own blocks into the same half with another layout; its copies
    must not start before the fetch's copies have landed (they would be overwritten)."""
    cfg = small_stream_cfg(n_layers=1, n_experts=12, n_slots=12, host_fraction=0.9)
    pool, dense, stats = build(cfg)
    try:
        from gpu_common import assert_slot_equals
        pool.poison_slots()
        pool.reset_page_table()
        side, main = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        for rep in range(3):
            a_set, b_set = [0, 1, 2, 3, 4, 5, 6, 7], [8, 9, 10, 11]
            pool.prefetch_host(0, a_set, side)
            pool.materialize(0, b_set, [0, 1, 2, 3], main)
            torch.cuda.synchronize()
            assert pool.device_errors() == 0
            for e, s in zip(b_set, [0, 1, 2, 3]):
                assert_slot_equals(pool, s, dense[0][0][e], dense[0][1][e])
            pool.prefetch_host(0, a_set, side)
            pool.materialize(0, a_set, [4, 5, 6, 7, 8, 9, 10, 11], main)
            torch.cuda.synchronize()
            for e, s in zip(a_set, [4, 5, 6, 7, 8, 9, 10, 11]):
                assert_slot_equals(pool, s, dense[0][0][e], dense[0][1][e])
    finally:
        pool.close()
