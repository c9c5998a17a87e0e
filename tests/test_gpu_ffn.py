"""GPU parity of the routed SwiGLU expert FFN against the FP64 oracle (variant B: the SwiGLU
product rounded to BF16 before the second product).  Tolerance: relative Frobenius error
<= 1e-3 (the target the build was given); the observed error is dominated by FP32
accumulation and by rare one-ulp disagreements of the BF16 rounding of h (about 1e-5)."""
import numpy as np
import pytest
import torch

from oracle import ffn as offn
from paper_2604_02715_amd import binding as B
from paper_2604_02715_amd import inputs

pytestmark = pytest.mark.gpu
TOL = 1e-3


def run_ffn_case(cfg, seed=0, waves=None, slot_perm=True, ids_override=None):
    from gpu_common import build_pool
    pool, dense = build_pool(cfg, seed=seed)
    try:
        w13, w2 = dense[0]
        x = inputs.activations(cfg, 0, seed=seed)
        ids, g = inputs.routing(cfg, 0, seed=seed)
        if ids_override is not None:
            ids = ids_override(ids)
        union = inputs.routed_union(ids)
        xd = x.cuda()
        idd = torch.from_numpy(ids).cuda()
        gd = torch.from_numpy(g).cuda()
        out = torch.full((cfg.tokens, cfg.hidden), 7.0, dtype=torch.float32, device="cuda")
        pool.reset_page_table()
        weights = lambda e: (inputs.bits_u16(w13[e]), inputs.bits_u16(w2[e]))
        if waves is None:
            assert len(union) <= cfg.n_slots
            perm = inputs.slot_permutation(cfg.n_slots, cfg.name, seed) if slot_perm else np.arange(cfg.n_slots)
            pool.materialize(0, union, perm[:len(union)])
            pool.expert_ffn(0, xd, idd, gd, out)
        else:
            first = True
            for w in waves(union):
                perm = inputs.slot_permutation(cfg.n_slots, cfg.name, seed, len(w))
                pool.materialize(0, w, perm[:len(w)])
                flags = B.FFN_SKIP_UNMAPPED | (0 if first else B.FFN_ACCUMULATE)
                pool.expert_ffn(0, xd, idd, gd, out, flags)
                pool.release(0, w)          # Sec. 3: the proxy releases what the block consumed
                first = False
        torch.cuda.synchronize()
        assert pool.device_errors() == 0
        want = offn.moe_ffn(inputs.bits_u16(x), ids, g, weights, round_h=True)
        exact = offn.moe_ffn(inputs.bits_u16(x), ids, g, weights, round_h=False)
        got = out.cpu().numpy()
        err = offn.rel_frobenius(got, want)
        print(cfg.name, "T", cfg.tokens, "K", cfg.top_k, "E", cfg.n_experts, "H", cfg.hidden, "F", cfg.ffn,
              "rel_frob vs B %.3e, vs A %.3e" % (err, offn.rel_frobenius(got, exact)), flush=True)
        assert np.isfinite(got).all()
        assert err <= TOL
        return got
    finally:
        pool.close()


def test_c1_tiny():
    run_ffn_case(inputs.CONFIGS["c1_tiny"])


@pytest.mark.parametrize("kw", [
    dict(tokens=1, top_k=1),                                   # a single pair
    dict(tokens=3, top_k=2, hidden=72, ffn=200),               # ragged strips and k tails
    dict(tokens=40, top_k=2, hidden=136, ffn=264, n_experts=4, n_slots=4),  # 8-column last strip
    dict(tokens=200, top_k=2, n_experts=3, n_slots=3),         # 133 rows per expert: LDS-tiled path
    dict(tokens=200, top_k=2, n_experts=3, n_slots=3, hidden=136, ffn=264),   # same rows, shapes the tiled path
                                                               # cannot take: two 96-row tiles per expert
    dict(tokens=256, top_k=2, hidden=320, ffn=448),            # about 64 rows per expert: 96-row tiles, both bodies
    dict(tokens=170, top_k=2, n_experts=4, n_slots=4),         # about 85 rows per expert: 128-row tiles
    dict(tokens=170, top_k=2, n_experts=4, n_slots=4, hidden=200, ffn=328),   # the same with ragged strips and k tails
    dict(tokens=230, top_k=2, n_experts=4, n_slots=4),         # about 115 rows per expert: 128-row tiles, some experts need two
    dict(tokens=120, top_k=2, routing="zipf"),                 # a popular expert overflows its 64-row tile
    dict(tokens=33, top_k=4, hidden=136, ffn=264, n_experts=5, n_slots=5),
    dict(tokens=16, top_k=8, hidden=256, ffn=4096),            # K split of the second product
    dict(tokens=700, top_k=2, n_experts=3, n_slots=3, hidden=192, ffn=320),   # LDS-tiled path, ragged edges
    dict(tokens=520, top_k=1, n_experts=2, n_slots=2, hidden=256, ffn=512),   # LDS-tiled path, full tiles + tail rows
    dict(tokens=300, top_k=1, n_experts=2, n_slots=2, hidden=256, ffn=1600),  # LDS-tiled path, K of the second product
                                                                              # split three ways (8, 8, 9 steps)
    dict(tokens=300, top_k=1, n_experts=2, n_slots=2, hidden=320, ffn=4096),  # split eight ways, ragged column tile
    dict(tokens=4400, top_k=2, n_experts=64, n_slots=64, hidden=64, ffn=128),  # 8800 pairs: more than the grouping kernel
                                                                               # keeps in registers between its passes
])
def test_shapes(kw):
    run_ffn_case(inputs.scaled(inputs.CONFIGS["c1_tiny"], **kw), seed=1)


@pytest.mark.parametrize("kw", [
    dict(tokens=700, top_k=2, n_experts=3, n_slots=3, hidden=192, ffn=320),
    dict(tokens=600, top_k=1, n_experts=2, n_slots=2, hidden=256, ffn=576),
    dict(tokens=600, top_k=1, n_experts=2, n_slots=2, hidden=64, ffn=128),    # one and two k steps, tile wider than N
])
def test_variants_of_the_tiled_kernels(monkeypatch, kw):
    """FLUXMOE_FFN_TILED_WAVES selects the variant of the LDS-tiled kernels: 2 (default) loads both
    operands straight into LDS with eight wavefronts, 1 does the same with four wavefronts of 128 x 128,
    8 and 4 stage them through registers with eight or four wavefronts.
    All accumulate over k in the same order, so they must agree to rounding."""
    cfg = inputs.scaled(inputs.CONFIGS["c1_tiny"], **kw)
    default = run_ffn_case(cfg, seed=1)
    for variant in ("8", "4", "2", "1"):
        monkeypatch.setenv("FLUXMOE_FFN_TILED_WAVES", variant)
        other = run_ffn_case(cfg, seed=1)
        assert offn.rel_frobenius(other, default) < 1e-5, variant


def test_more_experts_than_one_round_of_the_grouping_scans():
    """The grouping kernel scans the experts 1024 at a time and carries row and tile offsets from round to
    round: 1500 experts take two rounds."""
    run_ffn_case(inputs.scaled(inputs.CONFIGS["c1_tiny"], tokens=300, top_k=4, n_experts=1500, n_slots=1500,
                               hidden=64, ffn=128, routing="uniform"), seed=3)


@pytest.mark.parametrize("kw", [
    dict(tokens=20000, top_k=2, n_experts=1500, n_slots=1500, hidden=64, ffn=128, routing="uniform"),   # strip kernels, two scan rounds
    dict(tokens=33000, top_k=1, n_experts=4, n_slots=4, hidden=64, ffn=128),                            # LDS-tiled kernels
])
def test_batches_grouped_by_several_workgroups(kw):
    """More than 32768 pairs are counted and put in place by one workgroup per 8192 pairs around the
    workgroup that scans the experts; smaller batches by that workgroup alone."""
    run_ffn_case(inputs.scaled(inputs.CONFIGS["c1_tiny"], **kw), seed=7)


def test_all_pairs_on_one_expert_and_tiles_of_every_size_class():
    """Degenerate routings of the tile list: every token on expert 3 (two full 128-row tiles and a 44-row
    one with the strip kernels' largest tile forced), and expert row counts 1, 17, 33, 65, 97, 128, 129 that
    put a tile into every size class of the grouping kernel at once."""
    cfg = inputs.scaled(inputs.CONFIGS["c1_tiny"], tokens=300, top_k=1, n_experts=8, n_slots=8, hidden=136, ffn=264)
    run_ffn_case(cfg, seed=4, ids_override=lambda ids: np.full_like(ids, 3))
    counts = [1, 17, 33, 65, 97, 128, 129]
    cfg = inputs.scaled(cfg, tokens=sum(counts))
    def spread(ids):
        return np.repeat(np.arange(len(counts), dtype=ids.dtype), counts).reshape(ids.shape)
    run_ffn_case(cfg, seed=5, ids_override=spread)


def test_tile_order_of_the_tiled_gate_up_kernel_does_not_change_results(monkeypatch):
    """FLUXMOE_FFN_TILED_GROUP sets how many super-rows (4 row tiles of 256) of the LDS-tiled gate/up
    kernel share a column block in time.  It only renumbers workgroups: 12 row tiles (3 super-rows, the
    last group partial) by 18 column tiles (3 column blocks, the last partial) must come out bit for bit
    the same for every group size."""
    cfg = inputs.scaled(inputs.CONFIGS["c1_tiny"], tokens=3000, top_k=1, n_experts=2, n_slots=2, hidden=128, ffn=2304)
    monkeypatch.setenv("FLUXMOE_FFN_TILED_GROUP", "1")
    base = run_ffn_case(cfg, seed=2)
    for group in ("2", "3", "8"):
        monkeypatch.setenv("FLUXMOE_FFN_TILED_GROUP", group)
        assert np.array_equal(run_ffn_case(cfg, seed=2), base), group
    monkeypatch.delenv("FLUXMOE_FFN_TILED_GROUP")
    assert np.array_equal(run_ffn_case(cfg, seed=2), base)
    # FLUXMOE_FFN_TILED_PERSIST: 0 = one workgroup per tile number of the gate/up kernel, n = n x 256 workgroups
    # that each walk through several numbers (512 numbers here: two per workgroup with the default 1)
    for persist in ("0", "2"):
        monkeypatch.setenv("FLUXMOE_FFN_TILED_PERSIST", persist)
        assert np.array_equal(run_ffn_case(cfg, seed=2), base), persist
    monkeypatch.delenv("FLUXMOE_FFN_TILED_PERSIST")
    # the other variants of the tiled kernels at this size (more tile numbers than CUs); same sums in the same
    # order up to the grouping of partial products inside an MFMA
    for variant in ("1", "8", "4"):
        monkeypatch.setenv("FLUXMOE_FFN_TILED_WAVES", variant)
        assert offn.rel_frobenius(run_ffn_case(cfg, seed=2), base) < 1e-5, variant


@pytest.mark.parametrize("ffn", [640, 384, 2048])
def test_super_tile_shapes_of_the_walking_gate_up_kernel(ffn):
    """The workgroups of the LDS-tiled gate/up kernel walk through the tile numbers of super-tiles whose shape
    the launcher picks from the number of column tiles: 5 column tiles (ffn 640) give 16 x 2 super-tiles with
    one empty place per row, 3 (ffn 384) 8 x 4 with one empty column, 16 (ffn 2048) the 4 x 8 default.  9000
    rows in two experts are 37 row tiles: more tile numbers than workgroups in every shape, a partly filled
    last super-row, tail tiles with few rows."""
    cfg = inputs.scaled(inputs.CONFIGS["c1_tiny"], tokens=9000, top_k=1, n_experts=2, n_slots=2, hidden=128, ffn=ffn)
    run_ffn_case(cfg, seed=6)


def test_wave_mode_accumulates_to_the_single_shot_result():
    cfg = inputs.scaled(inputs.CONFIGS["c1_tiny"], n_slots=3)
    from oracle import paging
    a = run_ffn_case(cfg, waves=lambda u: paging.waves(u, 3))
    b = run_ffn_case(inputs.CONFIGS["c1_tiny"])
    assert offn.rel_frobenius(a, b) < 1e-6


def test_results_do_not_depend_on_slot_placement_and_are_reproducible():
    cfg = inputs.CONFIGS["c1_tiny"]
    a = run_ffn_case(cfg, slot_perm=True)
    b = run_ffn_case(cfg, slot_perm=False)
    c = run_ffn_case(cfg, slot_perm=True)
    assert np.array_equal(a, b) and np.array_equal(a, c)


def test_unmapped_expert_without_skip_flag_sets_the_error_word():
    from gpu_common import build_pool
    cfg = inputs.CONFIGS["c1_tiny"]
    pool, dense = build_pool(cfg)
    try:
        x = inputs.activations(cfg).cuda()
        ids, g = inputs.routing(cfg)
        out = torch.zeros((cfg.tokens, cfg.hidden), dtype=torch.float32, device="cuda")
        pool.reset_page_table()
        pool.materialize(0, [0, 1, 2], [0, 1, 2])
        pool.expert_ffn(0, x, torch.from_numpy(ids).cuda(), torch.from_numpy(g).cuda(), out)
        torch.cuda.synchronize()
        assert pool.device_errors() == 2
    finally:
        pool.close()


def test_shared_expert_added_on_top_of_the_routed_experts():
    """Configs 3 and 4 carry one shared expert: dense resident weights, every token, gate 1."""
    from gpu_common import build_pool
    cfg = inputs.scaled(inputs.CONFIGS["c1_tiny"], shared_expert=True, tokens=70, hidden=136, ffn=264)
    pool, dense = build_pool(cfg)
    try:
        w13, w2 = dense[0]
        s13, s2 = inputs.shared_expert_weights(cfg, 0)
        x = inputs.activations(cfg)
        ids, g = inputs.routing(cfg)
        out = torch.zeros((cfg.tokens, cfg.hidden), dtype=torch.float32, device="cuda")
        xd = x.cuda()
        s13d, s2d = s13.cuda(), s2.cuda()
        pool.reset_page_table()
        pool.materialize(0, np.arange(cfg.n_experts), np.arange(cfg.n_experts))
        pool.expert_ffn(0, xd, torch.from_numpy(ids).cuda(), torch.from_numpy(g).cuda(), out)
        pool.shared_expert_ffn(s13d, s2d, xd, out, B.FFN_ACCUMULATE)
        alone = torch.full_like(out, 5.0)
        pool.shared_expert_ffn(s13d, s2d, xd, alone)
        torch.cuda.synchronize()
        assert pool.device_errors() == 0
        xb = inputs.bits_u16(x)
        routed = offn.moe_ffn(xb, ids, g, lambda e: (inputs.bits_u16(w13[e]), inputs.bits_u16(w2[e])))
        T = cfg.tokens
        shared = offn.moe_ffn(xb, np.zeros((T, 1), dtype=np.int32), np.ones((T, 1), dtype=np.float32),
                              lambda e: (inputs.bits_u16(s13), inputs.bits_u16(s2)))
        assert offn.rel_frobenius(alone.cpu().numpy(), shared) <= TOL
        assert offn.rel_frobenius(out.cpu().numpy(), routed + shared) <= TOL
    finally:
        pool.close()


def test_mfma_probe_counts_what_it_claims():
    """The MFMA-only measurement aid: with all-ones operands every accumulator element grows by 16
    per MFMA (K = 16), so a lane's checksum is 16 accumulators x 16 elements x 16 x iters."""
    ones = torch.ones(32768, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(3 * 256, dtype=torch.float32, device="cuda")
    B.fluxmoe_mfma_probe(ones.data_ptr(), out.data_ptr(), 3, 5)
    torch.cuda.synchronize()
    assert torch.all(out == 16 * 16 * 16 * 5)


def test_empty_batch_and_fully_skipped_batch():
    """T = 0 enqueues nothing; with no expert mapped and the skip flag every pair is ignored: the
    result is zero, or the previous contents with the accumulate flag, and no error is flagged."""
    from gpu_common import build_pool
    cfg = inputs.CONFIGS["c1_tiny"]
    pool, dense = build_pool(cfg)
    try:
        x = inputs.activations(cfg).cuda()
        ids, g = inputs.routing(cfg)
        idd, gd = torch.from_numpy(ids).cuda(), torch.from_numpy(g).cuda()
        out = torch.full((cfg.tokens, cfg.hidden), 3.0, dtype=torch.float32, device="cuda")
        pool.reset_page_table()
        B.fluxmoe_expert_ffn(pool.ctx, 0, x.data_ptr(), 0, idd.data_ptr(), gd.data_ptr(), cfg.top_k,
                             pool.page_table.data_ptr(), out.data_ptr(), 0, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert torch.all(out == 3.0)
        pool.expert_ffn(0, x, idd, gd, out, B.FFN_SKIP_UNMAPPED | B.FFN_ACCUMULATE)
        torch.cuda.synchronize()
        assert torch.all(out == 3.0) and pool.device_errors() == 0
        pool.expert_ffn(0, x, idd, gd, out, B.FFN_SKIP_UNMAPPED)
        torch.cuda.synchronize()
        assert torch.all(out == 0.0) and pool.device_errors() == 0
    finally:
        pool.close()
