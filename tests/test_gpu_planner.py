"""Tensor-level offloading and restoration driven by the residency planner (Sec. 4.3): whatever
the planner moves between compressed GPU memory and pinned host memory, materialization must
still deliver the original bytes, and the planner's decisions on measured timings must be
the oracle model's."""
import numpy as np
import pytest
import torch

from oracle import planner as op
from paper_2604_02715_amd import binding as B
from paper_2604_02715_amd import harness, inputs

pytestmark = pytest.mark.gpu


def build(cfg):
    pool = harness.ExpertPool(cfg)
    dense, blobs = {}, {}
    for layer in range(cfg.n_layers):
        w13, w2 = harness.make_layer_on_host(cfg, layer)
        blob = pool.encode_layer(layer, w13, w2)
        pool.bind_layer(layer, blob, 0.0)
        dense[layer], blobs[layer] = (w13, w2), blob
    pool.bind_staging(2 * max(b.numel() for b in blobs.values()) + 8192)
    return pool, dense, blobs


def check_all_layers(pool, cfg, dense, timings=None):
    from gpu_common import assert_slot_equals
    ids = list(range(cfg.n_experts))
    for layer in range(cfg.n_layers):
        pool.poison_slots()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        pool.materialize(layer, ids, ids[::-1])
        b.record()
        torch.cuda.synchronize()
        if timings is not None:
            timings[layer] = a.elapsed_time(b)
        assert pool.device_errors() == 0
        for e, s in zip(ids, ids[::-1]):
            assert_slot_equals(pool, s, dense[layer][0][e], dense[layer][1][e])


def apply(pool, moves, blobs):
    for (layer, expert, type_, to_host) in moves:
        assert type_ in (1, 2)
        pool.set_tensor_backing(layer, type_, expert, bool(to_host), blobs[layer])


def test_offload_and_restore_steps_keep_materialization_exact():
    cfg = inputs.scaled(inputs.CONFIGS["c1_tiny"], n_layers=3, n_experts=8, n_slots=8)
    pool, dense, blobs = build(cfg)
    plan = B.fluxmoe_planner_create(cfg.n_layers, cfg.n_experts, 1, 0.9, 0.5)
    try:
        pool.reset_page_table()
        check_all_layers(pool, cfg, dense)
        # 6 steps of 4 down tensors empty the down stage, 2 more steps move 2 fused tensors each
        for step in range(8):
            moves = B.fluxmoe_planner_reclaim(plan)
            assert len(moves) == (4 if step < 6 else 2)
            apply(pool, moves, blobs)
            if step in (0, 5, 7):
                check_all_layers(pool, cfg, dense)
        _, on_host = B.fluxmoe_planner_state(plan, cfg.n_layers, cfg.n_experts)
        assert on_host[:, :, 1].all() and on_host[:, :, 0].sum() == 4
        for step in range(5):
            apply(pool, B.fluxmoe_planner_restore(plan), blobs)
        check_all_layers(pool, cfg, dense)
        while True:
            moves = B.fluxmoe_planner_restore(plan)
            if not moves:
                break
            apply(pool, moves, blobs)
        _, on_host = B.fluxmoe_planner_state(plan, cfg.n_layers, cfg.n_experts)
        assert not on_host.any()
        check_all_layers(pool, cfg, dense)
    finally:
        B.fluxmoe_planner_destroy(plan)
        pool.close()


def test_closed_loop_on_measured_load_times_follows_the_oracle():
    """Alg. 2 fed with materialization times measured on the device and a synthetic batch trace:
    a long queue (B_act << B_rem) makes it reclaim, a drained queue makes it restore."""
    cfg = inputs.scaled(inputs.CONFIGS["c1_tiny"], n_layers=2, n_experts=8, n_slots=8)
    pool, dense, blobs = build(cfg)
    plan = B.fluxmoe_planner_create(cfg.n_layers, cfg.n_experts, 2, 0.9, 0.25)
    ora = op.Planner(cfg.n_layers, cfg.n_experts, CI=2, AG=0.25)
    try:
        pool.reset_page_table()
        trace = [(4096, 64)] * 8 + [(64, 64)] * 2 + [(32, 32)] * 12
        seen = []
        for it, (B_rem, B_act) in enumerate(trace):
            timings = {}
            check_all_layers(pool, cfg, dense, timings)
            tau_load = [timings[l] for l in range(cfg.n_layers)]
            # forward latency: one tenth of the load time while the queue is long, a small
            # fraction once it has drained, so that rho moves from > 1 to < theta
            tau_fwd = sum(tau_load) * (0.1 if B_rem > B_act else 0.5)
            dec, moves = B.fluxmoe_planner_tick(plan, B_rem, B_act, tau_fwd, tau_load)
            action, rho, changed = ora.tick(B_rem, B_act, tau_fwd, tau_load)
            assert dec.action == action
            assert [(m[0], m[1], m[2]) for m in moves] == [tuple(c) for c in changed]
            apply(pool, moves, blobs)
            seen.append(dec.action)
        assert seen.count(B.PLAN_RECLAIM) == 4 and seen.count(B.PLAN_RESTORE) == 4
        _, on_host = B.fluxmoe_planner_state(plan, cfg.n_layers, cfg.n_experts)
        assert not on_host.any()
    finally:
        B.fluxmoe_planner_destroy(plan)
        pool.close()


def test_uncompressed_host_tensors_are_copied_not_decoded():
    """Tier 2 (Sec. 4.2's CPU offload backend: dense weights in pinned host memory): such tensors
    reach their slots bit for bit next to compressed host tensors and device-resident ones, with
    and without an explicit prefetch, and also when nothing at all is left to decode."""
    from gpu_common import assert_slot_equals
    cfg = inputs.scaled(inputs.CONFIGS["c1_tiny"], n_layers=2, n_experts=8, n_slots=8)
    pool, dense, blobs = build(cfg)
    try:
        pool.bind_staging(2 * cfg.n_experts * (cfg.sigma1 + cfg.sigma2) + 8192)
        pool.reset_page_table()
        w13, w2 = dense[0]
        raw = [((2, e), w2[e]) for e in (1, 4, 7)] + [((1, e), w13[e]) for e in (0, 4)]
        assert pool.place_tensors_raw_on_host(0, raw) == 3 * cfg.sigma2 + 2 * cfg.sigma1
        pool.place_tensors_on_host(0, blobs[0], [(2, 2), (1, 5)])          # compressed host tensors beside them
        ids = [4, 0, 7, 2, 5, 1, 3]
        slots = [0, 7, 3, 1, 6, 2, 5]
        side = torch.cuda.Stream()
        for prefetch in (False, True):
            pool.poison_slots()
            if prefetch:
                pool.prefetch_host(0, ids, side)
            pool.materialize(0, ids, slots)
            torch.cuda.synchronize()
            assert pool.device_errors() == 0
            for e, s in zip(ids, slots):
                assert_slot_equals(pool, s, w13[e], w2[e])
            table = pool.page_table.cpu().numpy().reshape(cfg.n_layers, cfg.n_experts)
            assert [table[0, e] for e in ids] == slots and table[0, 6] == -1
        # the other layer is untouched by the placement and still decodes from device memory
        check_all_layers(pool, cfg, dense)
        # every tensor of layer 1 uncompressed on the host: the call only copies and maps
        w13b, w2b = dense[1]
        allraw = [((2, e), w2b[e]) for e in range(cfg.n_experts)] + [((1, e), w13b[e]) for e in range(cfg.n_experts)]
        pool.place_tensors_raw_on_host(1, allraw)
        pool.poison_slots()
        order = list(range(cfg.n_experts))
        pool.materialize(1, order, order[::-1])
        torch.cuda.synchronize()
        assert pool.device_errors() == 0
        for e, s in zip(order, order[::-1]):
            assert_slot_equals(pool, s, w13b[e], w2b[e])
        table = pool.page_table.cpu().numpy().reshape(cfg.n_layers, cfg.n_experts)
        assert list(table[1]) == order[::-1] and (table[0] == -1).all()
        # back to device-resident compressed blocks
        for e in range(cfg.n_experts):
            for t in (1, 2):
                pool.set_tensor_backing(1, t, e, False, blobs[1])
        check_all_layers(pool, cfg, dense)
    finally:
        pool.close()
