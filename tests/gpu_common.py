"""Helpers for the GPU parity tests (import only inside tests marked gpu)."""
import numpy as np
import torch

from paper_2604_02715_amd import harness, inputs


def u16(t: torch.Tensor) -> np.ndarray:
    """Device/CPU int16 or bf16 tensor -> numpy uint16."""
    if t.dtype == torch.bfloat16:
        t = t.view(torch.int16)
    return t.cpu().numpy().view(np.uint16)


def build_pool(cfg, layers=None, seed=0, gen_device="cpu", host_fraction=0.0, max_tokens=None,
               max_top_k=None, weights=None):
    """Encode + bind the layers of cfg.  Returns (pool, {layer: (w13 CPU bf16, w2 CPU bf16)})."""
    pool = harness.ExpertPool(cfg, max_tokens=max_tokens, max_top_k=max_top_k)
    dense = {}
    for layer in (layers if layers is not None else range(cfg.n_layers)):
        if weights is not None:
            w13, w2 = weights[layer]
        else:
            w13, w2 = harness.make_layer_on_host(cfg, layer, seed, gen_device)
        blob = pool.encode_layer(layer, w13, w2)
        pool.bind_layer(layer, blob, host_fraction)
        dense[layer] = (w13, w2)
    return pool, dense


def assert_slot_equals(pool, slot, w13_e: torch.Tensor, w2_e: torch.Tensor):
    a = pool.slot13(slot)
    b = pool.slot2(slot)
    ref13 = w13_e.reshape(-1).view(torch.int16).to(a.device)
    ref2 = w2_e.reshape(-1).view(torch.int16).to(b.device)
    assert torch.equal(a, ref13), "type-1 slot %d differs from the original tensor" % slot
    assert torch.equal(b, ref2), "type-2 slot %d differs from the original tensor" % slot
