"""Full-size parity, in the launch configuration bench.py times.

Decoded weights: every byte of every materialized slot is compared (on the device) with the
original dense tensor, which is the definition of the lossless result; untouched slots must
keep their poison; the page table must equal the CPU placement model; blocks sampled from the
library's pool are decoded by the oracle and compared with the same slot bytes.
FFN: the oracle (FP64, h rounded to BF16) is evaluated on every token and every hidden column;
the gate is the relative Frobenius error over the whole output, and the worst single token must
meet the same bound.
"""
import numpy as np
import pytest
import torch

from oracle import codec, ffn as offn, paging
from paper_2604_02715_amd import binding as B
from paper_2604_02715_amd import inputs

pytestmark = pytest.mark.gpu
TOL = 1e-3


def check_slots(pool, dense, layer, ids, slots):
    w13, w2 = dense[layer]
    for e, s in zip(ids, slots):
        ref = w13[int(e)].reshape(-1).view(torch.int16).cuda()
        assert torch.equal(pool.slot13(int(s)), ref), "type-1 tensor of expert %d differs" % e
        ref = w2[int(e)].reshape(-1).view(torch.int16).cuda()
        assert torch.equal(pool.slot2(int(s)), ref), "type-2 tensor of expert %d differs" % e


def check_sampled_blocks_against_oracle(pool, blob, layer, ids, slots, n_samples=6, seed=0):
    rng = np.random.default_rng(seed)
    blocks = blob.numpy().reshape(-1, 4096)
    for _ in range(n_samples):
        i = int(rng.integers(len(ids)))
        d = int(rng.integers(1, 3))
        b0, nb = B.fluxmoe_tensor_blocks(pool.ctx, layer, d, int(ids[i]))
        k = int(rng.integers(nb))
        lens = B.fluxmoe_code_lengths(pool.ctx, layer, d)
        e0, n, parts = codec.decode_blocks(blocks[b0 + k:b0 + k + 1], lens)
        slot = pool.slot13(int(slots[i])) if d == 1 else pool.slot2(int(slots[i]))
        got = slot[int(e0[0]):int(e0[0]) + int(n[0])].cpu().numpy().view(np.uint16)
        assert np.array_equal(got, parts[0])
    # the block at the very end of a tensor (short tail)
    b0, nb = B.fluxmoe_tensor_blocks(pool.ctx, layer, 1, int(ids[0]))
    e0, n, parts = codec.decode_blocks(blocks[b0 + nb - 1:b0 + nb], B.fluxmoe_code_lengths(pool.ctx, layer, 1))
    got = pool.slot13(int(slots[0]))[int(e0[0]):int(e0[0]) + int(n[0])].cpu().numpy().view(np.uint16)
    assert np.array_equal(got, parts[0])


def run_full(cfg):
    from gpu_common import build_pool
    print("building", cfg.name, flush=True)
    pool = None
    try:
        from paper_2604_02715_amd import harness
        pool = harness.ExpertPool(cfg)
        w13, w2 = harness.make_layer_on_host(cfg, 0, 0, gen_device="cuda")
        blob = pool.encode_layer(0, w13, w2)
        pool.bind_layer(0, blob)
        dense = {0: (w13, w2)}
        x = inputs.activations(cfg)
        ids, g = inputs.routing(cfg)
        union = inputs.routed_union(ids)
        xd, idd, gd = x.cuda(), torch.from_numpy(ids).cuda(), torch.from_numpy(g).cuda()
        out = torch.full((cfg.tokens, cfg.hidden), 3.0, dtype=torch.float32, device="cuda")
        pool.poison_slots(0x7FC1)
        pool.reset_page_table()
        model = paging.PagedSlots(1, cfg.n_experts, cfg.n_slots, cfg.hidden, cfg.ffn, track_bytes=False)
        waves = paging.waves(union, cfg.n_slots)
        print(cfg.name, "union", len(union), "waves", [len(w) for w in waves], flush=True)
        for wi, w in enumerate(waves):
            slots = inputs.slot_permutation(cfg.n_slots, cfg.name, "full", wi)[:len(w)]
            model.materialize(0, w, slots, None, None)
            pool.materialize(0, w, slots)
            flags = (B.FFN_SKIP_UNMAPPED if len(waves) > 1 else 0) | (B.FFN_ACCUMULATE if wi else 0)
            pool.expert_ffn(0, xd, idd, gd, out, flags)
            torch.cuda.synchronize()
            assert pool.device_errors() == 0
            assert np.array_equal(pool.page_table.cpu().numpy(), model.page_table)
            check_slots(pool, dense, 0, w, slots)
            check_sampled_blocks_against_oracle(pool, blob, 0, w, slots, seed=wi)
            untouched = sorted(set(range(cfg.n_slots)) - set(int(s) for s in slots))
            if wi == 0 and untouched:
                s = untouched[0]
                assert bool((pool.slot13(s) == np.int16(0x7FC1)).all()) and bool((pool.slot2(s) == np.int16(0x7FC1)).all())
            if len(waves) > 1:
                model.release(0, w)
                pool.release(0, w)
        if cfg.shared_expert:                      # dense resident weights, all tokens, gate 1
            s13, s2 = inputs.shared_expert_weights(cfg, 0, device="cuda")
            pool.shared_expert_ffn(s13, s2, xd, out, B.FFN_ACCUMULATE)
        torch.cuda.synchronize()
        assert pool.device_errors() == 0
        # FFN: every token, every column
        weights = lambda e: (inputs.bits_u16(w13[e]), inputs.bits_u16(w2[e]))
        xb = inputs.bits_u16(x)
        want = offn.moe_ffn(xb, ids, g, weights, round_h=True)
        if cfg.shared_expert:
            s13h, s2h = inputs.bits_u16(s13.cpu()), inputs.bits_u16(s2.cpu())
            want = want + offn.moe_ffn(xb, np.zeros((cfg.tokens, 1), dtype=np.int32),
                                       np.ones((cfg.tokens, 1), dtype=np.float32), lambda e: (s13h, s2h), round_h=True)
        got = out.cpu().numpy()
        assert np.isfinite(got).all()
        err = offn.rel_frobenius(got, want)
        per_token = np.linalg.norm(got - want, axis=1) / np.linalg.norm(want, axis=1)
        print(cfg.name, "FFN rel. Frobenius error over all %d tokens = %.3e, worst token %d: %.3e"
              % (cfg.tokens, err, int(per_token.argmax()), float(per_token.max())), flush=True)
        assert err <= TOL
        assert float(per_token.max()) <= TOL
    finally:
        if pool is not None:
            pool.close()


def test_c2_mixtral_shaped_layer():
    run_full(inputs.CONFIGS["c2_mixtral"])


def test_c3_qwen3next_shaped_layer_two_waves():
    run_full(inputs.CONFIGS["c3_qwen3next"])


def test_c4_glm45_shaped_layer():
    run_full(inputs.CONFIGS["c4_glm45"])


def test_c2_mixtral_shaped_layer_prefill_batch():
    """The same layer with 1024 tokens (about 256 rows per expert): the LDS-tiled MFMA kernels at
    full size, the second product with its K split over two workgroups per tile."""
    run_full(inputs.scaled(inputs.CONFIGS["c2_mixtral"], tokens=1024))
