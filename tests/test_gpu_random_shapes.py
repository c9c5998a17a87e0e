"""GPU parity on seeded random shapes: the hand-picked cases of the other files aim at known edges
(ragged strips, k tails, tile classes, K splits); these draw experts, top-k, hidden, ffn, tokens,
routing law and row-tile size at random so that combinations nobody thought of are met too.
Same bars as everywhere: decode and placement bit for bit, FFN within 1e-3 relative Frobenius
of the FP64 oracle."""
import random

import pytest

from paper_2604_02715_amd import inputs
from test_gpu_ffn import run_ffn_case
from test_gpu_materialize import run_against_model

pytestmark = pytest.mark.gpu


def ffn_case(rnd):
    n_experts = rnd.choice([1, 2, 3, 5, 8, 17, 40, 130, 300])
    top_k = rnd.choice([k for k in (1, 2, 3, 4, 5, 8, 10, 12, 16, 20) if k <= n_experts])
    hidden = 8 * rnd.choice([1, 4, 8, 9, 17, 24, 32, 40, 64])
    ffn = 8 * rnd.choice([1, 3, 8, 16, 25, 33, 48, 64, 128])
    tokens = rnd.choice([1, 2, 7, 33, 100, 257, 600, 1500, 3000, 6000])
    while tokens * top_k * hidden * ffn > 3e9:               # keeps the FP64 oracle to a fraction of a second
        tokens = max(1, tokens // 2)
    routing = rnd.choice(["softmax", "zipf", "uniform"])
    m_tile = rnd.choice([None, None, "16", "32", "64", "96", "128", "256"])
    if m_tile == "256" and (hidden % 64 or ffn % 64):
        m_tile = None
    return dict(tokens=tokens, top_k=top_k, n_experts=n_experts, n_slots=n_experts, hidden=hidden, ffn=ffn,
                routing=routing), m_tile


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_ffn_on_random_shapes(monkeypatch, seed):
    rnd = random.Random(seed)
    for i in range(30):
        kw, m_tile = ffn_case(rnd)
        if m_tile:
            monkeypatch.setenv("FLUXMOE_FFN_MTILE", m_tile)
        else:
            monkeypatch.delenv("FLUXMOE_FFN_MTILE", raising=False)
        print("case", seed, i, kw, "row tile", m_tile, flush=True)
        run_ffn_case(inputs.scaled(inputs.CONFIGS["c1_tiny"], **kw), seed=100 * seed + i)


@pytest.mark.parametrize("seed", [21, 22])
def test_materialize_on_random_shapes_and_call_sequences(monkeypatch, seed):
    rnd = random.Random(seed)
    for i in range(25):
        n_experts = rnd.choice([1, 2, 3, 6])
        n_slots = n_experts + rnd.choice([0, 1, 3])
        hidden = 8 * rnd.choice([1, 2, 5, 9, 16, 41, 64])
        ffn = 8 * rnd.choice([1, 3, 8, 25, 57, 128])
        monkeypatch.setenv("FLUXMOE_DECODE_WAVES", rnd.choice(["4", "8", "16"]))
        monkeypatch.setenv("FLUXMOE_DECODE_BLOCKS_PER_WAVE", str(rnd.choice([1, 2, 3, 5])))
        cfg = inputs.scaled(inputs.CONFIGS["c1_tiny"], n_experts=n_experts, hidden=hidden, ffn=ffn,
                            n_slots=n_slots, n_layers=2)
        calls = []
        for _ in range(4):
            n = rnd.randint(0, min(n_experts, n_slots))
            ids = rnd.sample(range(n_experts), n)
            if rnd.random() < 0.2:
                calls.append((rnd.randrange(2), ids if n else None, "release"))     # None: the whole layer
            else:
                calls.append((rnd.randrange(2), ids, rnd.sample(range(n_slots), n)))
        print("case", seed, i, dict(n_experts=n_experts, n_slots=n_slots, hidden=hidden, ffn=ffn), calls, flush=True)
        run_against_model(cfg, calls, seed=100 * seed + i)
