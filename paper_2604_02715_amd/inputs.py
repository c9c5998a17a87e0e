"""Seeded synthetic inputs for the expert-materialization path.

This module only draws random inputs (expert weights, activations, routing, slot
assignments) with the shapes and value distributions of the workloads the paper
evaluates (Tab. "eval_model_memory": Mixtral-8x7B, Qwen3-Next-80B-A3B, GLM-4.5;
App. "Expert activation" for the routed-expert fractions).  It contains none of the
method's arithmetic: no codec, no paging, no FFN.  Both the CPU oracle's tests and the
HIP path's tests feed from here so that both sides see the same arrays.

Weight recipe: FP32 N(0, 0.02^2) times a per-row scale exp(N(0, 0.5^2)); optionally a
Bernoulli(1e-3) mask of entries multiplied by 16; rounded to BF16 (nearest-even).  The
exponent-byte entropy of this recipe (about 2.8 bits) reproduces the 32.1-32.5 % storage
saving the paper reports for real checkpoints (Sec. 4.2 "Compressed GPU backend").
"""
from __future__ import annotations

import dataclasses
import zlib

import numpy as np
import torch


@dataclasses.dataclass(frozen=True)
class LayerConfig:
    """One synthetic MoE layer workload."""

    name: str
    n_experts: int          # routed experts L per layer
    hidden: int             # H
    ffn: int                # F (per-expert intermediate size)
    tokens: int             # T decode tokens in the batch
    top_k: int              # K experts per token
    n_slots: int            # staging budget in experts
    routing: str            # "softmax" | "zipf" | "uniform"
    outliers: bool          # 0.1 % of entries x16
    shared_expert: bool = False
    n_layers: int = 1
    host_fraction: float = 0.0   # share of compressed blocks kept in pinned host DRAM

    @property
    def sigma1(self) -> int:     # bytes of one fused gate/up tensor [2][H][F]
        return 2 * self.hidden * self.ffn * 2

    @property
    def sigma2(self) -> int:     # bytes of one down tensor [F][H]
        return self.hidden * self.ffn * 2

    @property
    def pairs(self) -> int:
        return self.tokens * self.top_k


CONFIGS = {
    # tiny, CPU-quick
    "c1_tiny": LayerConfig("c1_tiny", 8, 256, 512, 64, 2, 8, "softmax", False),
    # Mixtral-8x7B-shaped layer
    "c2_mixtral": LayerConfig("c2_mixtral", 8, 4096, 14336, 256, 2, 8, "softmax", True),
    # Qwen3-Next-80B-A3B-shaped layer (256-slot pool: the routed union needs two waves)
    "c3_qwen3next": LayerConfig("c3_qwen3next", 512, 2048, 512, 256, 10, 256, "zipf", True,
                                shared_expert=True),
    # GLM-4.5-shaped layer
    "c4_glm45": LayerConfig("c4_glm45", 160, 5120, 1536, 512, 8, 160, "uniform", True,
                            shared_expert=True),
    # 16 GLM-4.5-shaped layers, 60/40 HBM/pinned-host split, 96 slots
    "c5_stream": LayerConfig("c5_stream", 160, 5120, 1536, 256, 8, 96, "zipf", True,
                             shared_expert=False, n_layers=16, host_fraction=0.40),
}


def scaled(cfg: LayerConfig, **kw) -> LayerConfig:
    """A copy of cfg with some fields replaced (reduced sizes for quick parity cases)."""
    return dataclasses.replace(cfg, **kw)


def _seed(*key) -> int:
    """Stable 63-bit seed from a tuple of ints/strings (independent sub-streams)."""
    text = "/".join(str(k) for k in key).encode()
    return (zlib.crc32(text) << 31) ^ zlib.adler32(text[::-1]) ^ 0x5DEECE66D


def _gen(device, *key) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(_seed(*key))
    return g


def weight_matrix(rows: int, cols: int, outliers: bool, device="cpu", *key) -> torch.Tensor:
    """One stored matrix [rows][cols] as a torch.bfloat16 tensor on `device`."""
    g = _gen(device, "w", *key)
    w = torch.randn(rows, cols, generator=g, device=device, dtype=torch.float32)
    w.mul_(0.02)
    row_scale = torch.exp(0.5 * torch.randn(rows, 1, generator=g, device=device,
                                            dtype=torch.float32))
    w.mul_(row_scale)
    if outliers:
        mask = torch.rand(rows, cols, generator=g, device=device) < 1e-3
        w = torch.where(mask, w * 16.0, w)
    return w.to(torch.bfloat16)


def expert_weights(cfg: LayerConfig, layer: int, expert: int, device="cpu", seed: int = 0):
    """(w13 [2][H][F], w2 [F][H]) BF16 for one routed expert.

    w13[0] is the gate projection, w13[1] the up projection; y = x @ W for all three.
    """
    H, F = cfg.hidden, cfg.ffn
    w1 = weight_matrix(H, F, cfg.outliers, device, cfg.name, seed, layer, expert, 1)
    w3 = weight_matrix(H, F, cfg.outliers, device, cfg.name, seed, layer, expert, 3)
    w2 = weight_matrix(F, H, cfg.outliers, device, cfg.name, seed, layer, expert, 2)
    return torch.stack([w1, w3], dim=0), w2


def shared_expert_weights(cfg: LayerConfig, layer: int, device="cpu", seed: int = 0):
    """Dense (never compressed) weights of the layer's shared expert, same shapes and recipe."""
    return expert_weights(cfg, layer, 1_000_000, device, seed)


def layer_weights(cfg: LayerConfig, layer: int, device="cpu", seed: int = 0,
                  out13: torch.Tensor | None = None, out2: torch.Tensor | None = None):
    """All routed experts of one layer: w13 [E][2][H][F], w2 [E][F][H] (BF16)."""
    E, H, F = cfg.n_experts, cfg.hidden, cfg.ffn
    if out13 is None:
        out13 = torch.empty(E, 2, H, F, dtype=torch.bfloat16, device=device)
    if out2 is None:
        out2 = torch.empty(E, F, H, dtype=torch.bfloat16, device=device)
    for e in range(E):
        a, b = expert_weights(cfg, layer, e, device, seed)
        out13[e].copy_(a)
        out2[e].copy_(b)
    return out13, out2


def bits_u16(t: torch.Tensor) -> np.ndarray:
    """The raw 16-bit patterns of a CPU BF16 tensor as a numpy uint16 array (no copy)."""
    assert t.dtype == torch.bfloat16 and t.device.type == "cpu"
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def activations(cfg: LayerConfig, layer: int = 0, device="cpu", seed: int = 0) -> torch.Tensor:
    """Token activations [T][H], N(0,1) rounded to BF16."""
    g = _gen(device, "x", cfg.name, seed, layer)
    return torch.randn(cfg.tokens, cfg.hidden, generator=g, device=device,
                       dtype=torch.float32).to(torch.bfloat16)


def routing(cfg: LayerConfig, layer: int = 0, seed: int = 0):
    """(topk_ids int32 [T][K], topk_w float32 [T][K]) as numpy arrays.

    softmax : logits N(0,1) over all experts, softmax, top-k (ties to the lower id),
              gates renormalised to sum 1 over the selected k.
    zipf    : popularity p_e ~ rank(e)^-1.1 with a seeded expert permutation; k distinct
              experts per token drawn proportionally (Gumbel top-k); gates = softmax of
              independent N(0,1) logits over the chosen k.
    uniform : k distinct experts uniformly at random; gates as for zipf.
    """
    rng = np.random.Generator(np.random.Philox(_seed("r", cfg.name, seed, layer)))
    T, K, E = cfg.tokens, cfg.top_k, cfg.n_experts
    if cfg.routing == "softmax":
        logits = rng.standard_normal((T, E))
        p = np.exp(logits - logits.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        ids = np.argsort(-p, axis=1, kind="stable")[:, :K]
        sel = np.take_along_axis(p, ids, axis=1)
        gates = sel / sel.sum(axis=1, keepdims=True)
    else:
        if cfg.routing == "zipf":
            rank = rng.permutation(E) + 1
            logp = -1.1 * np.log(rank.astype(np.float64))
        elif cfg.routing == "uniform":
            logp = np.zeros(E)
        else:
            raise ValueError(cfg.routing)
        gumbel = -np.log(-np.log(rng.random((T, E))))
        ids = np.argsort(-(logp[None, :] + gumbel), axis=1, kind="stable")[:, :K]
        gl = rng.standard_normal((T, K))
        gates = np.exp(gl - gl.max(axis=1, keepdims=True))
        gates /= gates.sum(axis=1, keepdims=True)
    return np.ascontiguousarray(ids, dtype=np.int32), np.ascontiguousarray(gates, dtype=np.float32)


def routed_union(topk_ids: np.ndarray) -> np.ndarray:
    """Sorted distinct expert ids that receive at least one token."""
    return np.unique(topk_ids.reshape(-1)).astype(np.int32)


def slot_permutation(n: int, *key) -> np.ndarray:
    """A seeded shuffle of range(n) (which slot each expert of a wave lands in)."""
    rng = np.random.Generator(np.random.Philox(_seed("s", *key)))
    return rng.permutation(n).astype(np.int32)


def adversarial_tensors() -> dict:
    """Small uint16 arrays (multiples of 64 elements) that stress the codec's corners."""
    rng = np.random.Generator(np.random.Philox(_seed("adv")))
    out = {}
    out["const_exponent"] = (np.uint16(0x3C00) | rng.integers(0, 128, 4096).astype(np.uint16))
    out["all_exponents"] = rng.integers(0, 1 << 16, 64 * 300).astype(np.uint16)
    special = np.array([0x0000, 0x8000, 0x7F80, 0xFF80, 0x7FC0, 0xFFC1, 0x0001, 0x807F,
                        0x7F7F, 0xFF7F, 0x0080, 0x3F80], dtype=np.uint16)
    out["specials"] = np.resize(special, 64 * 5)
    out["len64"] = rng.integers(0x3A00, 0x3E00, 64).astype(np.uint16)
    out["zeros"] = np.zeros(64 * 100, dtype=np.uint16)
    # two symbols only
    out["two_symbols"] = np.where(rng.random(64 * 64) < 0.9, 0x3C12, 0x4012).astype(np.uint16)
    # geometric exponent distribution: code lengths up to the limit and beyond
    geo = np.minimum(rng.geometric(0.5, 64 * 2048), 40).astype(np.uint16)
    out["geometric"] = ((100 + geo) << 7 | rng.integers(0, 128, geo.size).astype(np.uint16)
                        ).astype(np.uint16)
    return out
