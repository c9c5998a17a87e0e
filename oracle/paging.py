"""CPU model of slot placement and the page table: TEST INFRASTRUCTURE, not a product path.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.

What it follows.  PagedTensor (Sec. 4.1) gives the type-d tensor of expert l in layer i
the address  v0 + (i-1) S + (l-1) sigma_d  inside a reusable physical block, and states that
materialization only updates block contents.  This build replaces the layer term by a page
table lookup (expert -> staging slot), so the type-d tensor of an expert mapped to slot s
lives at  base_d + s * sigma_d.  Materializing expert e of layer i into slot s

  * makes slot s hold exactly the original dense bytes of both tensors of e,
  * sets page_table[i][e] = s,
  * sets the entry of whichever (layer, expert) owned slot s before to -1,
  * if e was mapped to another slot before, that slot becomes free,
  * leaves every other slot byte and page-table entry untouched.

Because decoding is lossless (Sec. 4.2), the slot contents need no codec to define.
"""
from __future__ import annotations

import numpy as np


class PagedSlots:
    def __init__(self, n_layers: int, n_experts: int, n_slots: int, hidden: int, ffn: int,
                 poison: int = 0x7FC1, track_bytes: bool = True):
        """track_bytes=False models only the page table and slot ownership (full-size layers,
        where the slot contents are compared on the device against the original tensors)."""
        self.n13 = 2 * hidden * ffn              # elements of a fused gate/up tensor
        self.n2 = hidden * ffn                   # elements of a down tensor
        self.track_bytes = track_bytes
        if track_bytes:
            self.slots13 = np.full((n_slots, self.n13), poison, dtype=np.uint16)
            self.slots2 = np.full((n_slots, self.n2), poison, dtype=np.uint16)
        self.page_table = np.full((n_layers, n_experts), -1, dtype=np.int32)
        self.owner = [None] * n_slots            # (layer, expert) or None

    def materialize(self, layer: int, expert_ids, dst_slots, dense13, dense2):
        """dense13(e) -> uint16 [n13], dense2(e) -> uint16 [n2] give the original weights."""
        expert_ids = [int(e) for e in expert_ids]
        dst_slots = [int(s) for s in dst_slots]
        assert len(set(expert_ids)) == len(expert_ids)
        assert len(set(dst_slots)) == len(dst_slots)
        for e, s in zip(expert_ids, dst_slots):
            old_slot = int(self.page_table[layer, e])
            if old_slot >= 0 and old_slot != s:
                self.owner[old_slot] = None
            prev = self.owner[s]
            if prev is not None and prev != (layer, e):
                self.page_table[prev[0], prev[1]] = -1
            if self.track_bytes:
                self.slots13[s] = np.asarray(dense13(e), dtype=np.uint16).reshape(-1)
                self.slots2[s] = np.asarray(dense2(e), dtype=np.uint16).reshape(-1)
            self.page_table[layer, e] = s
            self.owner[s] = (layer, e)

    def release(self, layer: int, expert_ids=None):
        """Sec. 3: after a layer's MoE block the proxy releases its experts: the mappings go,
        the slot bytes stay."""
        ids = range(self.page_table.shape[1]) if expert_ids is None else expert_ids
        for e in ids:
            s = int(self.page_table[layer, int(e)])
            if s >= 0:
                self.page_table[layer, int(e)] = -1
                self.owner[s] = None


def waves(union_ids, n_avail: int):
    """Cut a sorted routed union into consecutive waves of at most n_avail experts."""
    ids = sorted(int(e) for e in union_ids)
    return [ids[i:i + n_avail] for i in range(0, len(ids), n_avail)]


def paged_tensor_layout(N: int, L_r: int, hidden: int, ffn: int, g: int, n_uncompressed: int = 0):
    """Sec. 4.1 "Formal model" and "alignment analysis": for d = 1 (fused gate/up) and d = 2
    (down): sigma_d, A_d = L_r sigma_d, S_d = g ceil(A_d / g); virtual N S_d; physical blocks
    |U| + 2 per type; M_pad = (|U| + 2) sum_d (S_d - A_d)."""
    sigma = {2: hidden * ffn * 2}
    sigma[1] = 2 * sigma[2]
    A = {d: L_r * sigma[d] for d in (1, 2)}
    S = {d: g * -(-A[d] // g) for d in (1, 2)}
    return {"sigma": sigma, "A": A, "S": S,
            "virtual": N * (S[1] + S[2]),
            "physical": (n_uncompressed + 2) * (S[1] + S[2]),
            "M_pad": (n_uncompressed + 2) * ((S[1] - A[1]) + (S[2] - A[2]))}


def paged_tensor_address(v0: int, S: int, sigma: int, i: int, l: int) -> int:
    """addr = v0 + (i - 1) S + (l - 1) sigma with the paper's 1-based layer i and expert l."""
    return v0 + (i - 1) * S + (l - 1) * sigma


def reusable_block_of(i: int) -> int:
    """b_i = (i - 1) mod 2 for the paper's 1-based layer index."""
    return (i - 1) % 2
