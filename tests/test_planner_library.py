"""The library's residency planner (host logic, no GPU) against the oracle model of Sec. 4.3 /
Alg. 2, move by move, on seeded traces of (B_rem, B_act, tau_fwd, tau_load) signals."""
import math

import numpy as np
import pytest

from oracle import planner as op
from paper_2604_02715_amd import binding as B


def _oracle_moves(action, changed):
    out = []
    for c in changed:
        if c[0] == "layer":
            out.append((c[1], 0, 0, 1 if action == op.RECLAIM else 0))
        else:
            out.append((c[0], c[1], c[2], 1 if action == op.RECLAIM else 0))
    return out


def _state_of_oracle(p):
    pageable = np.array([0 if l in p.uncompressed else 1 for l in range(p.N)], dtype=np.uint8)
    on_host = np.zeros((p.N, p.L_r, 2), dtype=np.uint8)
    for (l, e, d) in p.on_host:
        on_host[l, e, d - 1] = 1
    return pageable, on_host


@pytest.mark.parametrize("N,L_r,AG,CI,theta,unc,seed", [
    (4, 4, 0.25, 16, 0.9, [], 1),
    (6, 8, 0.5, 4, 0.9, [1, 4], 2),
    (3, 5, 0.3, 1, 0.8, [0], 3),        # ceil(1.5) = 2 down, ceil(0.75) = 1 fused
    (5, 3, 1.0, 2, 0.95, [], 4),
    (2, 20, 0.75, 3, 0.9, [], 5),
])
def test_tick_trace_matches_oracle(N, L_r, AG, CI, theta, unc, seed):
    rng = np.random.Generator(np.random.Philox(seed))
    flags = [1 if l in unc else 0 for l in range(N)]
    lib_p = B.fluxmoe_planner_create(N, L_r, CI, theta, AG, flags)
    ora = op.Planner(N, L_r, theta=theta, AG=AG, CI=CI, uncompressed_layers=unc)
    try:
        B_rem = 4000
        phase = 0
        n_actions = {op.RECLAIM: 0, op.RESTORE: 0, op.KEEP: 0}
        for it in range(6000):
            if it % 500 == 0:
                phase = int(rng.integers(0, 3))             # pressure regime: reclaim / keep / restore
            B_act = int(rng.integers(0, 257)) if rng.random() > 0.05 else 0
            B_act = min(B_act, B_rem)
            tau_load = rng.uniform(0.5, 2.0, N) if rng.random() > 0.02 else np.zeros(N)
            target = (3.0, 0.95, 0.3)[phase] * rng.uniform(0.8, 1.25)
            tau_fwd = target * tau_load.sum() * (B_act / B_rem if B_act else 1.0) if tau_load.sum() else 1.0
            dec, moves = B.fluxmoe_planner_tick(lib_p, B_rem, B_act, tau_fwd, tau_load)
            action, rho, changed = ora.tick(B_rem, B_act, tau_fwd, list(tau_load))
            assert dec.action == action, (it, dec.action, action)
            if action in (op.KEEP, op.RECLAIM, op.RESTORE):
                n_actions[action] += 1
                if math.isinf(rho):
                    assert math.isinf(dec.rho)
                else:
                    assert dec.rho == pytest.approx(rho, rel=1e-12)
            assert moves == _oracle_moves(action, changed), (it, moves, changed)
            if rng.random() < 0.01 and B_rem > 0:
                B_rem = max(0, B_rem - int(rng.integers(1, 40)))
        assert min(n_actions.values()) > 0, n_actions      # the trace exercised all three rules
        pg, oh = B.fluxmoe_planner_state(lib_p, N, L_r)
        pg_o, oh_o = _state_of_oracle(ora)
        assert np.array_equal(pg, pg_o) and np.array_equal(oh, oh_o)
        dec, _ = B.fluxmoe_planner_tick(lib_p, 0, 0, 1.0, None)
        assert dec.action == B.PLAN_DONE
    finally:
        B.fluxmoe_planner_destroy(lib_p)


def test_full_reclaim_then_full_restore_round_trip():
    N, L_r, AG = 5, 6, 0.4
    lib_p = B.fluxmoe_planner_create(N, L_r, 1, 0.9, AG, [0, 1, 0, 0, 1])
    ora = op.Planner(N, L_r, AG=AG, CI=1, uncompressed_layers=[1, 4])
    try:
        steps = 0
        while True:
            m = B.fluxmoe_planner_reclaim(lib_p)
            assert m == _oracle_moves(op.RECLAIM, ora.reclaim())
            if not m:
                break
            steps += 1
        pg, oh = B.fluxmoe_planner_state(lib_p, N, L_r)
        assert pg.all() and oh.all()                        # everything pageable and host-backed
        # 2 layer steps + ceil(30 / ceil(2.4)) down steps + ceil(30 / ceil(1.2)) fused steps
        assert steps == 2 + 10 + 15
        for _ in range(steps):
            m = B.fluxmoe_planner_restore(lib_p)
            assert m and m == _oracle_moves(op.RESTORE, ora.restore())
        assert B.fluxmoe_planner_restore(lib_p) == []
        pg, oh = B.fluxmoe_planner_state(lib_p, N, L_r)
        assert list(pg) == [1, 0, 1, 1, 0] and not oh.any()
    finally:
        B.fluxmoe_planner_destroy(lib_p)


@pytest.mark.parametrize("N,L,G,AG,released", [
    (32, 8, 2, 0.25, 24), (32, 8, 2, 0.75, 54), (89, 160, 8, 0.25, 4600), (48, 512, 4, 0.5, 9216),
])
def test_library_replays_released_counts_of_the_paper(N, L, G, AG, released):
    """Tab. 'exp5-settings': the released down-projection tensors are whole steps of ceil(AG L_r)."""
    L_r = L // G
    lib_p = B.fluxmoe_planner_create(N, L_r, 16, 0.9, AG)
    try:
        step = math.ceil(AG * L_r)
        assert B.fluxmoe_planner_max_moves(lib_p) == step
        total = 0
        for _ in range(released // (G * step)):
            m = B.fluxmoe_planner_reclaim(lib_p)
            assert len(m) == step and all(t == 2 and h == 1 for (_, _, t, h) in m)
            total += len(m)
        assert total * G == released
        _, oh = B.fluxmoe_planner_state(lib_p, N, L_r)
        per_layer = oh[:, :, 1].sum(axis=1)
        assert int(per_layer.sum()) == total and per_layer.max() - per_layer.min() <= 1
        assert not oh[:, :, 0].any()
    finally:
        B.fluxmoe_planner_destroy(lib_p)


def test_argument_errors():
    with pytest.raises(B.FluxmoeError):
        B.fluxmoe_planner_create(0, 4)
    with pytest.raises(B.FluxmoeError):
        B.fluxmoe_planner_create(2, 4, adjustment_granularity=1.5)
    with pytest.raises(B.FluxmoeError):
        B.fluxmoe_planner_create(2, 4, theta=-0.1)
    p = B.fluxmoe_planner_create(2, 4)
    try:
        with pytest.raises(B.FluxmoeError):
            B.fluxmoe_planner_tick(p, 10, 5, -1.0, [1.0, 1.0])
        with pytest.raises(B.FluxmoeError):
            B.fluxmoe_planner_tick(p, 10, 5, 1.0, [1.0, float("nan")])
    finally:
        B.fluxmoe_planner_destroy(p)


def test_balanced_split_matches_oracle():
    rng = np.random.Generator(np.random.Philox(11))
    cases = [(7.0, 1.0, 8), (100.0, 0.0, 16), (1.0, 1.0, 4), (2800.0, 84.5, 160), (400.0, 50.0, 20)]
    cases += [(float(rng.uniform(50, 5000)), float(rng.uniform(0, 3000)), int(rng.integers(1, 513)))
              for _ in range(500)]
    for bg, bc, L_r in cases:
        x, nd, nf = B.fluxmoe_balanced_split(bg, bc, L_r)
        xo, ndo, nfo, _ = op.balanced_split(bg, bc, L_r)
        assert x == pytest.approx(xo, rel=1e-15) and (nd, nf) == (ndo, nfo), (bg, bc, L_r)
    with pytest.raises(B.FluxmoeError):
        B.fluxmoe_balanced_split(0.0, 1.0, 8)
    with pytest.raises(B.FluxmoeError):
        B.fluxmoe_balanced_split(1.0, 1.0, 0)
