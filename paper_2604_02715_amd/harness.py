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
        ffn_ws = B.fluxmoe_ffn_workspace_bytes(self.ctx, T, K, cfg.shared_expert)
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
        self.tensor_copies = {}

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

    def set_tensor_backing(self, layer, type_, expert, to_host: bool, blob: torch.Tensor):
        """Carry out one tensor move of the residency planner (Sec. 4.3): copy the tensor's blocks
        out of the layer blob (CPU uint8) into pinned host or device memory and re-point the
        library at that copy.  The previous copy is dropped after a device synchronisation."""
        Bk = self.cfg_block_bytes
        first, nb = B.fluxmoe_tensor_blocks(self.ctx, layer, type_, expert)
        part = blob[first * Bk:(first + nb) * Bk]
        if to_host:
            copy = torch.empty(nb * Bk, dtype=torch.uint8, pin_memory=True)
            copy.copy_(part)
        else:
            copy = part.to(self.device)
        B.fluxmoe_set_tensor_backing(self.ctx, layer, type_, expert, 1 if to_host else 0, copy.data_ptr())
        torch.cuda.synchronize()
        self.tensor_copies[(layer, type_, expert)] = copy

    def place_tensors_on_host(self, layer, blob: torch.Tensor, tensors):
        """Whole-tensor host placement of a bound layer (Sec. 4.2: the bandwidth-balanced split is
        realised with whole down-projection tensors): the listed (type, expert) tensors are packed
        into one pinned buffer, down tensors first, each group by ascending expert, so that the
        staging copy of a routed set is a few long DMAs.  Returns the pinned bytes."""
        Bk = self.cfg_block_bytes
        order = sorted(tensors, key=lambda te: (-te[0], te[1]))
        ranges = [B.fluxmoe_tensor_blocks(self.ctx, layer, t, e) for (t, e) in order]
        total = sum(nb for _, nb in ranges) * Bk
        if total == 0:
            return 0
        pinned = torch.empty(total, dtype=torch.uint8, pin_memory=True)
        at = 0
        for (t, e), (first, nb) in zip(order, ranges):
            pinned[at:at + nb * Bk].copy_(blob[first * Bk:(first + nb) * Bk])
            B.fluxmoe_set_tensor_backing(self.ctx, layer, t, e, 1, pinned.data_ptr() + at)
            at += nb * Bk
        self.host_blobs[layer] = pinned
        return total

    def place_tensors_raw_on_host(self, layer, dense):
        """Uncompressed host placement (the CPU offload backend as Sec. 4.2 states it): `dense` is a
        list of ((type, expert), BF16 tensor); the tensors' bytes are packed into one pinned buffer
        and the library is pointed at them (tier 2: fetched by DMA, copied into the slot, never
        decoded).  Returns the pinned bytes."""
        order = sorted(dense, key=lambda kv: (-kv[0][0], kv[0][1]))
        total = sum(t.numel() * 2 for _, t in order)
        if total == 0:
            return 0
        pinned = torch.empty(total, dtype=torch.uint8, pin_memory=True)
        at = 0
        for (t, e), w in order:
            nbytes = w.numel() * 2
            pinned[at:at + nbytes].copy_(w.contiguous().reshape(-1).view(torch.uint8))
            B.fluxmoe_set_tensor_backing(self.ctx, layer, t, e, B.TIER_HOST_RAW, pinned.data_ptr() + at)
            at += nbytes
        self.host_blobs[("raw", layer)] = pinned
        return total

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

    def materialize_two_streams(self, layer, expert_ids, dst_slots, stream, stream_type2):
        B.fluxmoe_materialize_two_streams(self.ctx, layer, expert_ids, self.page_table.data_ptr(), dst_slots,
                                          _sptr(stream), _sptr(stream_type2))

    def release(self, layer, expert_ids=None, stream=None):
        B.fluxmoe_release(self.ctx, layer, expert_ids, self.page_table.data_ptr(), _sptr(stream))

    def expert_ffn(self, layer, tokens, topk_ids, topk_w, out, flags=0, stream=None):
        T, K = topk_ids.shape
        assert tokens.dtype == torch.bfloat16 and tokens.is_contiguous() and out.dtype == torch.float32
        assert topk_ids.dtype == torch.int32 and topk_w.dtype == torch.float32
        B.fluxmoe_expert_ffn(self.ctx, layer, tokens.data_ptr(), T, topk_ids.data_ptr(),
                             topk_w.data_ptr(), K, self.page_table.data_ptr(), out.data_ptr(), flags,
                             _sptr(stream))

    def shared_expert_ffn(self, w13, w2, tokens, out, flags=0, stream=None):
        assert w13.dtype == torch.bfloat16 and w13.is_contiguous() and w2.is_contiguous()
        B.fluxmoe_shared_expert_ffn(self.ctx, w13.data_ptr(), w2.data_ptr(), tokens.data_ptr(),
                                    tokens.shape[0], out.data_ptr(), flags, _sptr(stream))

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


class StreamingProxy:
    """The forward proxy of Sec. 3 over all layers of a pool, with Alg. 1's stream layout.

    Layer l materializes into the slot half l & 1 (two reusable halves, Sec. 4.1) on the load
    stream while layer l - 1 runs its FFN on the inference stream; host-tier blocks of layer
    l + 2 are fetched on the copy stream as soon as layer l's last materialize has been issued.
    A routed union larger than one half is cut into waves (materialize, FFN with
    skip-unmapped/accumulate, release).  Ordering between the streams is entirely the
    library's (events inside fluxmoe_materialize / fluxmoe_expert_ffn / fluxmoe_prefetch_host).
    """

    def __init__(self, pool: ExpertPool, routings, xs, outs, seed=0, streams=None):
        cfg = pool.cfg
        self.pool, self.cfg = pool, cfg
        self.xs, self.outs = xs, outs
        self.ids = [torch.from_numpy(r[0]).to(pool.device) for r in routings]
        self.gates = [torch.from_numpy(r[1]).to(pool.device) for r in routings]
        self.half = cfg.n_slots // 2
        self.plan = []                      # per layer: list of (expert ids, slots)
        for layer, (ids_np, _) in enumerate(routings):
            union = sorted(int(e) for e in inputs.routed_union(ids_np))
            base = (layer & 1) * self.half
            waves = []
            for w0 in range(0, len(union), self.half):
                w = union[w0:w0 + self.half]
                perm = inputs.slot_permutation(self.half, cfg.name, seed, layer, w0)[:len(w)]
                waves.append((np.asarray(w, dtype=np.int32), (base + perm).astype(np.int32)))
            self.plan.append((np.asarray(union, dtype=np.int32), waves))
        # The device has few hardware queues per process; streams created later can share one, and
        # then an event wait in one stream holds back the other.  A caller that builds several
        # proxies passes the same three streams to all of them.
        self.load_stream, self.infer_stream, self.copy_stream = streams or (
            torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())

    def run_pass(self, layer_done_events=None, single_stream=False, ffn_delay_cycles=0, after_wave=None):
        """Issue one pass over all layers.  single_stream=True puts everything on the
        inference stream in program order (the reference schedule for hazard checks).
        after_wave(layer, wave index, expert ids, slots), if given, is called after a wave's FFN has
        been issued and before its release (a test synchronises there and inspects the slots).
        ffn_delay_cycles > 0 holds the inference stream back before every FFN (a bounded
        spin kernel), which widens the window in which a missing write-after-read wait would
        let the next materialize overwrite slots that the FFN has not read yet."""
        p, n_layers = self.pool, self.cfg.n_layers
        ls = self.infer_stream if single_stream else self.load_stream
        cs = self.infer_stream if single_stream else self.copy_stream
        host = bool(p.host_blobs)
        if host:
            p.prefetch_host(0, self.plan[0][0], cs)
            if n_layers > 1:
                p.prefetch_host(1, self.plan[1][0], cs)
        for layer in range(n_layers):
            union, waves = self.plan[layer]
            for wi, (w, slots) in enumerate(waves):
                p.materialize(layer, w, slots, ls)
                if host and wi == len(waves) - 1 and layer + 2 < n_layers:
                    p.prefetch_host(layer + 2, self.plan[layer + 2][0], cs)
                flags = (B.FFN_SKIP_UNMAPPED if len(waves) > 1 else 0) | (B.FFN_ACCUMULATE if wi else 0)
                if ffn_delay_cycles:
                    with torch.cuda.stream(self.infer_stream):
                        torch.cuda._sleep(int(ffn_delay_cycles))
                p.expert_ffn(layer, self.xs[layer], self.ids[layer], self.gates[layer], self.outs[layer],
                             flags, self.infer_stream)
                if after_wave is not None:
                    after_wave(layer, wi, w, slots)
                p.release(layer, w, self.infer_stream)
            if layer_done_events is not None:
                layer_done_events[layer].record(self.infer_stream)
