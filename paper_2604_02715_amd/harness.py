"""Device-memory plumbing around the C ABI for tests, smoke() and bench.py.

PyTorch is used here only to own device / pinned memory and streams; every computation is a
call into libfluxmoe.so through `binding`.  The harness plays the paper's forward proxy
(Sec. 3): it decides which experts to materialize into which slots and when to run the FFN.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from . import inputs


class ExpertPool:
    """One context + its device arenas for a LayerConfig."""

    def __init__(self, cfg: inputs.LayerConfig, device="cuda:0", max_tokens=None, max_top_k=None,
                 n_threads=16):
        self.cfg = cfg
        self.device = torch.device(device)
        self.n_threads = n_threads
        self.ctx = B.fluxmoe_create(cfg.n_layers, cfg.n_experts, cfg.hidden, cfg.ffn, cfg.n_slots)
        self.sizes = B.fluxmoe_query_sizes(self.ctx)
        T = max_tokens or cfg.tokens
        K = max_top_k or cfg.top_k
        ffn_ws = B.fluxmoe_ffn_workspace_bytes(self.ctx, T, K)
        self.ws_bytes = int(self.sizes.pool_workspace_bytes + ffn_ws)
        dev = self.device
        self.slots13 = torch.empty(self.sizes.slots13_bytes // 2, dtype=torch.int16, device=dev)
        self.slots2 = torch.empty(self.sizes.slots2_bytes // 2, dtype=torch.int16, device=dev)
        self.workspace = torch.zeros(self.ws_bytes, dtype=torch.uint8, device=dev)
        self.page_table = torch.full((cfg.n_layers, cfg.n_experts), -1, dtype=torch.int32, device=dev)
        B.fluxmoe_bind_arenas(self.ctx, self.slots13.data_ptr(), self.slots2.data_ptr(),
                              self.workspace.data_ptr(), self.ws_bytes)
        self.hbm_blobs = {}
        self.host_blobs = {}
        self.staging = None
        self.blob_bytes = {}

    def close(self):
        if self.ctx is not None:
            torch.cuda.synchronize()
            B.fluxmoe_destroy(self.ctx)
            self.ctx = None

    # ------------------------------------------------------------------ pool set-up
    def poison_slots(self, pattern=0x7FC1):
        v = np.array(pattern, dtype=np.uint16).view(np.int16).item()
        self.slots13.fill_(v)
        self.slots2.fill_(v)

    def encode_layer(self, layer, w13_host: torch.Tensor, w2_host: torch.Tensor, keep_host_copy=False):
        """w13_host/w2_host: CPU BF16 tensors [E][2][H][F], [E][F][H].  Returns the blob (CPU uint8)."""
        assert w13_host.device.type == "cpu" and w13_host.is_contiguous() and w2_host.is_contiguous()
        cap = int(self.sizes.layer_blob_bound)
        blob = torch.empty(cap, dtype=torch.uint8)
        used = B.fluxmoe_encode_pool(self.ctx, layer, w13_host.data_ptr(), w2_host.data_ptr(),
                                     blob.data_ptr(), cap, self.n_threads)
        self.blob_bytes[layer] = used
        return blob[:used]

    def bind_layer(self, layer, blob: torch.Tensor, host_fraction=0.0, check=True):
        """Split the blob between pinned host (leading blocks) and HBM (the rest) and bind."""
        Bk = self.cfg_block_bytes
        n_blocks = blob.numel() // Bk
        n_host = int(np.ceil(host_fraction * n_blocks - 1e-12)) if host_fraction > 0 else 0
        host_ptr = None
        if n_host:
            pinned = torch.empty(n_host * Bk, dtype=torch.uint8, pin_memory=True)
            pinned.copy_(blob[: n_host * Bk])
            self.host_blobs[layer] = pinned
            host_ptr = pinned.data_ptr()
        dev_part = blob[n_host * Bk:].to(self.device)
        self.hbm_blobs[layer] = dev_part
        B.fluxmoe_bind_layer(self.ctx, layer, dev_part.data_ptr() if dev_part.numel() else None,
                             n_host, host_ptr, blob.data_ptr() if check else None)
        return n_blocks, n_host

    @property
    def cfg_block_bytes(self):
        return 4096

    def bind_staging(self, nbytes):
        self.staging = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        B.fluxmoe_bind_staging(self.ctx, self.staging.data_ptr(), nbytes)

    # ------------------------------------------------------------------ hot path
    def reset_page_table(self, stream=None):
        B.fluxmoe_reset_page_table(self.ctx, self.page_table.data_ptr(), _sptr(stream))

    def prefetch_host(self, layer, expert_ids, stream=None):
        B.fluxmoe_prefetch_host(self.ctx, layer, expert_ids, _sptr(stream))

    def materialize(self, layer, expert_ids, dst_slots, stream=None):
        B.fluxmoe_materialize(self.ctx, layer, expert_ids, self.page_table.data_ptr(), dst_slots,
                              _sptr(stream))

    def release(self, layer, expert_ids=None, stream=None):
        B.fluxmoe_release(self.ctx, layer, expert_ids, self.page_table.data_ptr(), _sptr(stream))

    def expert_ffn(self, layer, tokens, topk_ids, topk_w, out, flags=0, stream=None):
        T, K = topk_ids.shape
        assert tokens.dtype == torch.bfloat16 and tokens.is_contiguous() and out.dtype == torch.float32
        assert topk_ids.dtype == torch.int32 and topk_w.dtype == torch.float32
        B.fluxmoe_expert_ffn(self.ctx, layer, tokens.data_ptr(), T, topk_ids.data_ptr(),
                             topk_w.data_ptr(), K, self.page_table.data_ptr(), out.data_ptr(), flags,
                             _sptr(stream))

    def device_errors(self):
        return B.fluxmoe_device_errors(self.ctx)

    # ------------------------------------------------------------------ views for checks
    def slot13(self, s) -> torch.Tensor:
        n = self.sizes.sigma1 // 2
        return self.slots13[s * n:(s + 1) * n]

    def slot2(self, s) -> torch.Tensor:
        n = self.sizes.sigma2 // 2
        return self.slots2[s * n:(s + 1) * n]


def _sptr(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return stream


def make_layer_on_host(cfg: inputs.LayerConfig, layer=0, seed=0, gen_device="cpu"):
    """Synthetic layer weights as CPU BF16 tensors (generated on gen_device, copied back)."""
    w13, w2 = inputs.layer_weights(cfg, layer, device=gen_device, seed=seed)
    return w13.cpu().contiguous(), w2.cpu().contiguous()
