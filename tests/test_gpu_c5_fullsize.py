"""Config 5 at its full size: 16 GLM-4.5-shaped layers (160 experts of 5120 x 1536), 60 % of every
layer's compressed blocks in HBM and 40 % in pinned host memory fetched on a side stream, 96 staging
slots as two halves of 48, 256 tokens top-8 with Zipf routing, three streams (Sec. 3 sliding window,
Sec. 4.2 host tier, Alg. 1).

Pass 1 runs the forward proxy's schedule and stops after every wave: every slot the wave materialized is
compared on the device with the original dense tensor (the definition of the lossless result), the page
table with the CPU placement model, and blocks sampled from both tiers of the layer's pool with what the
oracle decoded from the same pool bytes.  Pass 2 runs all 16 layers overlapped without stopping; its FFN
outputs must equal pass 1's bit for bit (the kernels are deterministic, so any slot overwritten before it
was read, or read before it was written, in any layer shows up here), and the FFN output of sampled tokens
of every layer must be within 1e-3 relative Frobenius error of the FP64 oracle.  All 16 layers are
distinct (no weight templates are reused).
"""
import time

import numpy as np
import pytest
import torch

from oracle import codec, ffn as offn, paging
from paper_2604_02715_amd import binding as B
from paper_2604_02715_amd import harness, inputs

pytestmark = pytest.mark.gpu
TOL = 1e-3
SAMPLE_TOKENS = 3
SAMPLE_BLOCKS = 4


def test_c5_streaming_all_layers_full_size():
    cfg = inputs.CONFIGS["c5_stream"]
    t0 = time.time()
    pool = harness.ExpertPool(cfg)
    try:
        routings = [inputs.routing(cfg, layer) for layer in range(cfg.n_layers)]
        rng = np.random.default_rng(11)
        samples = {}                      # layer -> list of (type, expert, e0, expected uint16 array)
        n_host_total = 0
        for layer in range(cfg.n_layers):
            w13, w2 = harness.make_layer_on_host(cfg, layer, 0, gen_device="cuda")
            blob = pool.encode_layer(layer, w13, w2)
            n_blocks, n_host = pool.bind_layer(layer, blob, cfg.host_fraction, check=(layer == 0))
            assert n_host == int(np.ceil(cfg.host_fraction * n_blocks - 1e-12))
            n_host_total += n_host
            # oracle decode of sampled blocks of routed experts: half from the host-tier prefix of the
            # blob (down tensors come first), half from the HBM part (fused tensors of higher experts)
            blocks = blob.numpy().reshape(-1, 4096)
            union = inputs.routed_union(routings[layer][0])
            picks = []
            for i in range(SAMPLE_BLOCKS):
                d = 2 if i % 2 == 0 else 1
                e = int(union[-1 - (i // 2)]) if d == 1 else int(rng.choice(union))
                b0, nb = B.fluxmoe_tensor_blocks(pool.ctx, layer, d, e)
                k = int(rng.integers(nb)) if i < 2 else nb - 1          # also the short last block
                lens = B.fluxmoe_code_lengths(pool.ctx, layer, d)
                e0, n, parts = codec.decode_blocks(blocks[b0 + k:b0 + k + 1], lens)
                picks.append((d, e, int(e0[0]), parts[0].copy(), (b0 + k) < n_host))
            assert any(p[4] for p in picks) and not all(p[4] for p in picks), "samples must cover both tiers"
            samples[layer] = picks
            del w13, w2, blob, blocks
            print("layer %d encoded and bound (%.0f s)" % (layer, time.time() - t0), flush=True)
        pool.bind_staging(2 * (n_host_total // cfg.n_layers + 64) * 4096 + 8192)

        xs_host = [inputs.activations(cfg, layer) for layer in range(cfg.n_layers)]
        xs = [x.cuda() for x in xs_host]
        outs = [torch.full((cfg.tokens, cfg.hidden), float("nan"), dtype=torch.float32, device="cuda")
                for _ in range(cfg.n_layers)]
        proxy = harness.StreamingProxy(pool, routings, xs, outs)
        assert proxy.half == 48 and all(len(waves) >= 2 for _, waves in proxy.plan)
        pool.poison_slots()
        pool.reset_page_table()
        torch.cuda.synchronize()

        # ---------------- pass 1: stop after every wave and check
        model = paging.PagedSlots(cfg.n_layers, cfg.n_experts, cfg.n_slots, cfg.hidden, cfg.ffn, track_bytes=False)
        state = {"layer": -1, "w13": None, "w2": None, "checked": 0, "sampled": 0}
        sel_tokens = {layer: np.sort(np.random.default_rng(100 + layer).choice(cfg.tokens, SAMPLE_TOKENS, replace=False))
                      for layer in range(cfg.n_layers)}
        oracle_w = {}                     # (layer, expert) -> (w13 bits, w2 bits) of experts the sampled tokens use

        def after_wave(layer, wi, w, slots):
            torch.cuda.synchronize()
            assert pool.device_errors() == 0
            if state["layer"] != layer:
                state["w13"], state["w2"] = None, None
                state["w13"], state["w2"] = inputs.layer_weights(cfg, layer, device="cuda")
                state["layer"] = layer
            model.materialize(layer, w, slots, None, None)
            assert np.array_equal(pool.page_table.cpu().numpy(), model.page_table), "page table, layer %d wave %d" % (layer, wi)
            needed = set(int(e) for e in routings[layer][0][sel_tokens[layer]].reshape(-1))
            for e, s_ in zip(w, slots):
                e, s_ = int(e), int(s_)
                assert torch.equal(pool.slot13(s_), state["w13"][e].reshape(-1).view(torch.int16)), \
                    "layer %d expert %d: type-1 slot %d differs from the original" % (layer, e, s_)
                assert torch.equal(pool.slot2(s_), state["w2"][e].reshape(-1).view(torch.int16)), \
                    "layer %d expert %d: type-2 slot %d differs from the original" % (layer, e, s_)
                state["checked"] += 1
                for d, se, e0, want, _host in samples[layer]:
                    if se == e:
                        view = pool.slot13(s_) if d == 1 else pool.slot2(s_)
                        got = view[e0:e0 + want.size].cpu().numpy().view(np.uint16)
                        assert np.array_equal(got, want), "layer %d expert %d type %d block at %d vs oracle" % (layer, e, d, e0)
                        state["sampled"] += 1
                if e in needed:
                    oracle_w[(layer, e)] = (inputs.bits_u16(state["w13"][e].cpu()), inputs.bits_u16(state["w2"][e].cpu()))
            model.release(layer, w)
            if wi == 0:
                print("layer %d wave 0 checked (%.0f s)" % (layer, time.time() - t0), flush=True)

        proxy.run_pass(after_wave=after_wave)
        torch.cuda.synchronize()
        state["w13"], state["w2"] = None, None
        assert pool.device_errors() == 0
        assert state["checked"] == sum(len(u) for u, _ in proxy.plan)
        assert state["sampled"] == SAMPLE_BLOCKS * cfg.n_layers
        assert (pool.page_table.cpu().numpy() == -1).all()
        first = [o.cpu().numpy().copy() for o in outs]

        # ---------------- FFN of sampled tokens of every layer against the oracle
        for layer in range(cfg.n_layers):
            sel = sel_tokens[layer]
            ids, g = routings[layer]
            want = offn.moe_ffn(inputs.bits_u16(xs_host[layer])[sel], ids[sel], g[sel],
                                lambda e: oracle_w[(layer, e)], round_h=True)
            err = offn.rel_frobenius(first[layer][sel], want)
            print("layer %d FFN rel. Frobenius error on tokens %s = %.3e" % (layer, sel.tolist(), err), flush=True)
            assert np.isfinite(first[layer]).all()
            assert err <= TOL
        oracle_w.clear()

        # ---------------- pass 2 and 3: overlapped, no stops; same bits in every layer
        for rep in range(2):
            for o in outs:
                o.fill_(float("nan"))
            pool.poison_slots()
            torch.cuda.synchronize()
            proxy.run_pass()
            torch.cuda.synchronize()
            assert pool.device_errors() == 0
            for layer in range(cfg.n_layers):
                assert np.array_equal(outs[layer].cpu().numpy(), first[layer]), \
                    "overlapped pass %d changed the FFN output of layer %d" % (rep, layer)
            assert (pool.page_table.cpu().numpy() == -1).all()
        print("config 5 full size done (%.0f s)" % (time.time() - t0), flush=True)
    finally:
        pool.close()
