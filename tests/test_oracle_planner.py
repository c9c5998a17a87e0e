"""Pins for the planner model against what the paper prints (Sec. 4.3, Alg. 2, Exp#5 and
Tab. 'exp5-settings')."""
import math

import pytest

from oracle import planner as op


def test_control_signal_definitions():
    # tau_eff = (B_rem / B_act) tau_fwd; tau_load = sum over layers; rho = ratio
    assert op.Planner.rho(512, 256, 10.0, [2.0, 3.0]) == pytest.approx(4.0)
    assert op.Planner.rho(256, 256, 10.0, [0.0, 0.0]) == math.inf          # +inf for zero load


def test_rules_dead_zone_and_guards():
    p = op.Planner(4, 8, CI=1)
    load = [1.0] * 4
    assert p.tick(512, 256, 5.0, load)[0] == op.RECLAIM       # rho = 2.5 > 1 and B_act < B_rem
    assert p.tick(256, 256, 5.0, load)[0] == op.KEEP          # rho > 1 but nobody is waiting
    assert p.tick(512, 256, 1.9, load)[0] == op.KEEP          # rho = 0.95: inside [theta, 1]
    assert p.tick(512, 256, 1.7, load)[0] == op.RESTORE       # rho = 0.85 < 0.9
    assert p.tick(512, 256, 1.7, load)[0] == op.KEEP          # nothing left to restore
    assert p.tick(512, 0, 1.7, load)[0] == op.SKIP            # B_act = 0: interval skipped
    assert p.tick(0, 0, 1.7, load)[0] == op.DONE              # B_rem = 0 ends the loop


def test_control_interval():
    p = op.Planner(2, 4, CI=16)
    acts = [p.tick(10, 5, 100.0, [1.0, 1.0])[0] for _ in range(48)]
    assert [i for i, a in enumerate(acts) if a != op.SKIP] == [15, 31, 47]


@pytest.mark.parametrize("model,N,L,G,cells", [
    # (AG, released tensors over all GPUs) from Tab. 'exp5-settings', CI = 16 rows and AG = 0.25 rows
    ("glm45", 89, 160, 8, [(0.25, 9200), (0.25, 4600), (0.25, 2320), (0.25, 1200), (0.50, 9200), (0.75, 9960), (1.00, 11680)]),
    ("qwen3next", 48, 512, 4, [(0.25, 9216), (0.25, 4864), (0.25, 2432), (0.25, 1280), (0.50, 9216), (0.75, 9600), (1.00, 9728)]),
    ("mixtral", 32, 8, 2, [(0.25, 42), (0.25, 24), (0.25, 18), (0.25, 14), (0.50, 40), (0.75, 54), (1.00, 72)]),
])
def test_released_tensor_counts_of_the_paper_are_whole_steps(model, N, L, G, cells):
    """Every cell of the table is a whole number of reclamation steps of ceil(AG L_r) down
    tensors per rank; replaying that many steps releases exactly that many tensors, all of
    them down projections, spread over the layers."""
    L_r = L // G
    for AG, released in cells:
        step = math.ceil(AG * L_r)
        assert released % (G * step) == 0, (model, AG, released)
        steps = released // (G * step)
        p = op.Planner(N, L_r, AG=AG)
        for _ in range(steps):
            moved = p.reclaim()
            assert len(moved) == step and all(d == op.DOWN for (_, _, d) in moved)
        assert len(p.on_host) * G == released
        vols = [p.cpu_volume(l) for l in range(N)]
        assert max(vols) - min(vols) <= 1                     # smallest-CPU-volume-first spreads evenly


def test_mixtral_twelve_steps_release_24_tensors():
    """App. text under Tab. 'exp5-settings': L_r = 4, each of the 12 AG = 0.25 adjustments
    offloads one down-projection tensor per rank: 24 tensors over two ranks."""
    p = op.Planner(32, 4, AG=0.25)
    for _ in range(12):
        assert len(p.reclaim()) == 1
    assert 2 * len(p.on_host) == 24


def test_released_memory_matches_the_papers_compressed_sizes():
    """Released memory = sum of compressed-copy sizes (Sec. 4.3); with the 32.1-32.5 % saving of
    Sec. 4.2 the table's GB follow from the tensor counts."""
    for H, F, count, gb in ((5120, 1536, 4600, 48.8), (2048, 512, 4864, 6.9), (4096, 14336, 24, 1.9)):
        dense = H * F * 2
        lo, hi = count * dense * (1 - 0.325) / 1e9, count * dense * (1 - 0.321) / 1e9
        assert lo * 0.98 <= gb <= hi * 1.02


def test_selection_order_and_stage_change():
    p = op.Planner(3, 4, AG=0.5)                               # steps of 2 down tensors, then 1 fused
    assert p.reclaim() == [(2, 3, op.DOWN), (1, 3, op.DOWN)]   # equal volumes: larger layer first
    assert p.reclaim() == [(0, 3, op.DOWN), (2, 2, op.DOWN)]   # layer 0 had the smallest volume
    for _ in range(4):
        p.reclaim()
    assert all((l, e, op.DOWN) in p.on_host for l in range(3) for e in range(4))
    assert p.reclaim() == [(2, 3, op.FUSED)]                   # down tensors exhausted: ceil(AG L_r / 2)
    assert p.reclaim() == [(1, 3, op.FUSED)]
    assert p.restore() == [(1, 3, op.FUSED)]                   # restoration reverses the sequence
    assert p.restore() == [(2, 3, op.FUSED)]
    assert p.restore() == [(0, 0, op.DOWN), (1, 0, op.DOWN)]   # last down step, last pick first
    assert len(p.on_host) == 10


def test_layer_stage_comes_first():
    p = op.Planner(4, 2, AG=0.5, uncompressed_layers=[0, 2])
    assert p.reclaim() == [("layer", 2)]
    assert p.reclaim() == [("layer", 0)]
    assert p.reclaim() == [(3, 1, op.DOWN)]
    assert p.restore() == [(3, 1, op.DOWN)]
    assert p.restore() == [("layer", 0)] and 0 in p.uncompressed


def test_balanced_split_formula_bound_and_mixtral_case():
    """Sec. 4.2: x_bw = beta_cpu / (beta_gpu + beta_cpu); ceil(3 L_r x_bw) down tensors;
    0 <= x_i - x_bw < 1 / (3 L_r).  Exp#3's caption: Mixtral keeps 87.5 % on the compressed GPU
    backend, i.e. a CPU share of 1/8, which is 3 whole down tensors of a rank holding 8
    experts' shards and leaves 1.233 GB of the 1.409 GB per-GPU layer to decode."""
    x, n_down, n_fused, xr = op.balanced_split(7.0, 1.0, 8)
    assert x == 0.125 and (n_down, n_fused) == (3, 0) and xr == 0.125
    per_gpu = 8 * 3 * 4096 * 14336 * 2 / 2
    assert (1 - xr) * per_gpu / 1e9 == pytest.approx(1.233, abs=1e-3)
    import random
    rnd = random.Random(7)
    for _ in range(2000):
        bg, bc, L_r = rnd.uniform(50, 5000), rnd.uniform(1, 100), rnd.randint(1, 512)
        x, n_down, n_fused, xr = op.balanced_split(bg, bc, L_r)
        assert x * (bg + bc) == pytest.approx(bc)             # equal backend times: x / bc = (1 - x) / bg
        assert x / bc == pytest.approx((1 - x) / bg)
        if x < 1 / 3:
            assert n_fused == 0 and -1e-12 <= xr - x < 1 / (3 * L_r)
    assert op.balanced_split(100.0, 0.0, 16)[1:3] == (0, 0)
    assert op.balanced_split(1.0, 1.0, 4)[1:3] == (4, 1)      # x = 1/2: 6 units = 4 down + 1 fused
