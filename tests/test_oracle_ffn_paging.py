"""Pins for the FP64 FFN oracle and the slot/page-table model."""
import math

import numpy as np
import pytest
import torch

from oracle import ffn, paging
from paper_2604_02715_amd import inputs


def f64_to_bf16_bits(x):
    return inputs.bits_u16(torch.tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16))


# ------------------------------------------------------------------ numeric helpers
def test_bf16_widening_is_exact_and_rounding_matches_nearest_even():
    bits = np.array([0x3F80, 0xBF80, 0x4000, 0x3DCD, 0x0000, 0x8000], dtype=np.uint16)
    assert list(ffn.bf16_bits_to_f64(bits)) == [1.0, -1.0, 2.0, 0.10009765625, 0.0, -0.0]
    # hand values: 8 significant bits
    assert ffn.round_to_bf16(np.array([2.1931757358]))[0] == 2.1875
    assert ffn.round_to_bf16(np.array([5.2847824678]))[0] == 5.28125
    # ties go to the even significand: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert ffn.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert ffn.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    # against an independent implementation (torch's float32 -> bfloat16 cast)
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(200000) * np.exp(rng.standard_normal(200000) * 3)).astype(np.float32)
    want = torch.tensor(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(ffn.round_to_bf16(x.astype(np.float64)), want)


def test_silu_closed_form_values():
    assert ffn.silu(np.array([0.0]))[0] == 0.0
    assert abs(ffn.silu(np.array([1.0]))[0] - 1 / (1 + math.exp(-1))) < 1e-16
    assert abs(ffn.silu(np.array([-2.0]))[0] + 2 / (1 + math.exp(2))) < 1e-16


# ------------------------------------------------------------------ tiny case by hand
def test_hand_computed_two_by_two():
    """x = [1, 2]; W1 = I; W3 = ones; W2 = I.  a = [1, 2], b = [3, 3],
    h = 3*silu([1, 2]) = [2.1931757358, 5.2847824678]; BF16(h) = [2.1875, 5.28125]."""
    x = f64_to_bf16_bits([[1.0, 2.0]])
    w13 = f64_to_bf16_bits([[[1, 0], [0, 1]], [[1, 1], [1, 1]]])
    w2 = f64_to_bf16_bits([[1, 0], [0, 1]])
    ids = np.array([[0]], dtype=np.int32)
    g = np.array([[1.0]], dtype=np.float32)
    A = ffn.moe_ffn(x, ids, g, lambda e: (w13, w2), round_h=False)
    B = ffn.moe_ffn(x, ids, g, lambda e: (w13, w2), round_h=True)
    assert np.allclose(A, [[3 / (1 + math.exp(-1)), 6 / (1 + math.exp(-2))]], rtol=0, atol=1e-15)
    assert np.array_equal(B, [[2.1875, 5.28125]])
    # a transposed operand would change this one: W2 not symmetric
    w2t = f64_to_bf16_bits([[0, 1], [0, 0]])               # y = h @ W2 -> [0, h0]
    B2 = ffn.moe_ffn(x, ids, g, lambda e: (w13, w2t), round_h=True)
    assert np.array_equal(B2, [[0.0, 2.1875]])
    w13n = f64_to_bf16_bits([[[0, 1], [0, 0]], [[1, 1], [1, 1]]])   # a = x @ W1 = [0, 1]
    B3 = ffn.moe_ffn(x, ids, g, lambda e: (w13n, w2), round_h=False)
    assert np.allclose(B3, [[0.0, 3 / (1 + math.exp(-1))]], rtol=0, atol=1e-15)


# ------------------------------------------------------------------ properties
def small_problem(seed=0, T=12, H=32, F=48, E=5, K=2):
    cfg = inputs.scaled(inputs.CONFIGS["c1_tiny"], n_experts=E, hidden=H, ffn=F, tokens=T, top_k=K)
    w13, w2 = inputs.layer_weights(cfg, 0, seed=seed)
    w13, w2 = inputs.bits_u16(w13), inputs.bits_u16(w2)
    x = inputs.bits_u16(inputs.activations(cfg, seed=seed))
    ids, g = inputs.routing(cfg, seed=seed)
    return cfg, w13, w2, x, ids, g


def test_single_expert_reduces_to_matmul_chain():
    cfg, w13, w2, x, ids, g = small_problem(K=1)
    ids[:] = 3
    g[:] = 1.0
    out = ffn.moe_ffn(x, ids, g, lambda e: (w13[e], w2[e]), round_h=False)
    X = torch.tensor(ffn.bf16_bits_to_f64(x))
    W1, W3 = (torch.tensor(ffn.bf16_bits_to_f64(w13[3][i])) for i in (0, 1))
    W2 = torch.tensor(ffn.bf16_bits_to_f64(w2[3]))
    want = (torch.nn.functional.silu(X @ W1) * (X @ W3)) @ W2
    assert np.allclose(out, want.numpy(), rtol=1e-12, atol=1e-15)


def test_zero_gate_projection_gives_zero_and_gates_are_linear():
    cfg, w13, w2, x, ids, g = small_problem()
    z13 = w13.copy(); z13[:, 0] = 0
    assert not ffn.moe_ffn(x, ids, g, lambda e: (z13[e], w2[e])).any()
    base = ffn.moe_ffn(x, ids, g, lambda e: (w13[e], w2[e]))
    assert np.allclose(ffn.moe_ffn(x, ids, 2 * g, lambda e: (w13[e], w2[e])), 2 * base,
                       rtol=1e-14, atol=0)


def test_token_permutation_equivariance_and_wave_split():
    cfg, w13, w2, x, ids, g = small_problem(T=16, E=6, K=3)
    base = ffn.moe_ffn(x, ids, g, lambda e: (w13[e], w2[e]))
    perm = np.random.default_rng(1).permutation(16)
    out = ffn.moe_ffn(x[perm], ids[perm], g[perm], lambda e: (w13[e], w2[e]))
    assert np.allclose(out, base[perm], rtol=1e-13, atol=1e-18)
    # two waves over disjoint expert subsets accumulate to the single-shot result
    acc = ffn.moe_ffn(x, ids, g, lambda e: (w13[e], w2[e]), mapped={0, 1, 2})
    acc = ffn.moe_ffn(x, ids, g, lambda e: (w13[e], w2[e]), mapped={3, 4, 5}, out=acc)
    assert np.allclose(acc, base, rtol=1e-13, atol=1e-18)


def test_rounding_h_costs_about_bf16_half_ulp():
    cfg, w13, w2, x, ids, g = small_problem(T=32, H=64, F=128)
    A = ffn.moe_ffn(x, ids, g, lambda e: (w13[e], w2[e]), round_h=False)
    B = ffn.moe_ffn(x, ids, g, lambda e: (w13[e], w2[e]), round_h=True)
    err = ffn.rel_frobenius(B, A)
    assert 3e-4 < err < 4e-3              # uniform error within +-2^-9 relative per element


# ------------------------------------------------------------------ routing generators
def test_routing_generators_have_the_stated_structure():
    for name in ("c1_tiny", "c3_qwen3next", "c4_glm45"):
        cfg = inputs.CONFIGS[name]
        ids, g = inputs.routing(cfg)
        assert ids.shape == (cfg.tokens, cfg.top_k) and g.dtype == np.float32
        assert all(len(set(r)) == cfg.top_k for r in ids)
        assert np.allclose(g.sum(axis=1), 1.0, atol=1e-6) and (g > 0).all()
        assert ids.min() >= 0 and ids.max() < cfg.n_experts
    # App. 'Expert activation': > 70 % of Qwen3-Next's experts active at batch 256
    u = inputs.routed_union(inputs.routing(inputs.CONFIGS["c3_qwen3next"])[0])
    assert 0.70 * 512 < len(u) <= 512 and len(u) > 256
    u = inputs.routed_union(inputs.routing(inputs.CONFIGS["c4_glm45"])[0])
    assert len(u) == 160


# ------------------------------------------------------------------ page-table model
def test_placement_model():
    H, F, E, S = 8, 16, 6, 4
    ps = paging.PagedSlots(2, E, S, H, F)
    d13 = lambda e: np.full(2 * H * F, 100 + e, dtype=np.uint16)
    d2 = lambda e: np.full(H * F, 200 + e, dtype=np.uint16)
    ps.materialize(0, [4, 1], [2, 0], d13, d2)
    assert list(ps.page_table[0]) == [-1, 0, -1, -1, 2, -1]
    assert (ps.slots13[2] == 104).all() and (ps.slots2[0] == 201).all()
    assert (ps.slots13[1] == 0x7FC1).all() and (ps.slots2[3] == 0x7FC1).all()
    # layer 1 takes slot 2: layer 0's expert 4 loses its mapping
    ps.materialize(1, [5], [2], d13, d2)
    assert ps.page_table[0, 4] == -1 and ps.page_table[1, 5] == 2 and ps.page_table[0, 1] == 0
    # moving an expert frees its old slot and keeps a single mapping
    ps.materialize(0, [1], [3], d13, d2)
    assert ps.page_table[0, 1] == 3 and ps.owner[0] is None and ps.owner[3] == (0, 1)
    # swapping two experts' slots inside one call
    ps.materialize(0, [1, 2], [1, 3], d13, d2)
    assert ps.page_table[0, 1] == 1 and ps.page_table[0, 2] == 3
    assert (ps.slots13[1] == 101).all() and (ps.slots13[3] == 102).all()
    assert paging.waves([5, 1, 9, 3, 7], 2) == [[1, 3], [5, 7], [9]]
    # release: mappings go, bytes stay, unmapped ids are ignored
    ps.release(0, [1, 5])
    assert ps.page_table[0, 1] == -1 and ps.owner[1] is None and (ps.slots13[1] == 101).all()
    assert ps.page_table[0, 2] == 3
    ps.release(0)
    assert (ps.page_table[0] == -1).all() and ps.page_table[1, 5] == 2
