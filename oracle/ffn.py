"""FP64 oracle of the routed SwiGLU expert FFN: TEST INFRASTRUCTURE, not a product path.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.

What it follows.  Each routed expert owns a fused gate/up-projection tensor and a
down-projection tensor (Sec. 4.1 "Formal model": tensor types d = 1, 2).  The paper runs an
unchanged fused-MoE kernel on them (Sec. 5), so the block's meaning is the standard one:

    a = x W1,  b = x W3,  h = silu(a) * b,  y = h W2,  out_t = sum_k g_{t,k} y_{e_{t,k}}

with silu(a) = a / (1 + exp(-a)), W13 stored [2][H][F] (gate first, then up), W2 stored
[F][H], all BF16 values widened exactly to FP64.

Two variants.  A: no intermediate rounding.  B: h is rounded to BF16 (nearest-even) before
the second product, everything else FP64; this is the point where a BF16-input matrix-core
kernel must round, and it is the variant the GPU result is held to (relative Frobenius
error <= 1e-3).  The paper is silent on the intermediate precision.
"""
from __future__ import annotations

import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """uint16 BF16 patterns -> float64 (exact)."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest BF16 value (ties to even), returned as float64.

    BF16 keeps 8 significant bits: x = m * 2^ex with m in [0.5, 1); rounding m * 256 to the
    nearest integer (ties to even, numpy's rint) gives the 8-bit significand.  Values whose
    magnitude is below the BF16 normal range are not expected here (h is O(1e-4..1e1)).
    """
    x = np.asarray(x, dtype=np.float64)
    m, ex = np.frexp(x)
    return np.ldexp(np.rint(m * 256.0) / 256.0, ex)


def silu(a: np.ndarray) -> np.ndarray:
    return a / (1.0 + np.exp(-a))


def expert_ffn(x: np.ndarray, w13: np.ndarray, w2: np.ndarray, round_h: bool) -> np.ndarray:
    """One expert on a batch of rows.  x [M][H], w13 [2][H][F], w2 [F][H], all float64."""
    a = x @ w13[0]
    b = x @ w13[1]
    h = silu(a) * b
    if round_h:
        h = round_to_bf16(h)
    return h @ w2


def moe_ffn(x_bits: np.ndarray, topk_ids: np.ndarray, topk_w: np.ndarray, weights,
            round_h: bool = True, mapped=None, out: np.ndarray | None = None) -> np.ndarray:
    """out [T][H] float64.

    x_bits   uint16 [T][H] BF16 activations
    topk_ids int [T][K], topk_w float32 [T][K]
    weights  callable e -> (w13_bits uint16 [2][H][F], w2_bits uint16 [F][H])
    mapped   optional set of expert ids; pairs routed to other experts are skipped (a wave
             of a slot budget smaller than the routed union); `out` is then accumulated into
    """
    x = bf16_bits_to_f64(x_bits)
    T, H = x.shape
    if out is None:
        out = np.zeros((T, H), dtype=np.float64)
    ids = np.asarray(topk_ids)
    g = np.asarray(topk_w, dtype=np.float32).astype(np.float64)
    for e in np.unique(ids):
        if mapped is not None and int(e) not in mapped:
            continue
        t_idx, k_idx = np.nonzero(ids == e)
        w13_bits, w2_bits = weights(int(e))
        y = expert_ffn(x[t_idx], bf16_bits_to_f64(w13_bits), bf16_bits_to_f64(w2_bits), round_h)
        # a token lists an expert at most once, so t_idx has no repeats
        out[t_idx] += g[t_idx, k_idx][:, None] * y
    return out


def rel_frobenius(a: np.ndarray, ref: np.ndarray) -> float:
    a = np.asarray(a, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(a - ref) / np.linalg.norm(ref))
