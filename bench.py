#!/usr/bin/env python3
"""Benchmark of the expert-materialization hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input: materialize the
routed experts of a layer from the compressed HBM pool into their staging slots (decode +
paged scatter + page-table update), then run the routed SwiGLU expert FFN on them.  The
default workload is the Mixtral-8x7B-shaped layer (8 experts, H 4096, F 14336, 256 decode
tokens, top-2; all 8 experts materialized every step).  Prints ONE JSON line.

  value      dense BF16 bytes materialized per second of whole-step time (GB/s, GB = 1e9 B),
             the paper's throughput definition (Sec. 6.3, Exp#3) applied to the whole step
  roofline   the decode kernel against HBM peak: algorithmic bytes (compressed blocks read +
             dense bytes written) per launch / mean launch duration from HIP events recorded
             around the kernel on its own stream
  cpu_baseline  the CPU oracle's decoder timed here on a bounded sample of the same pool
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="c2_mixtral", help="c1_tiny | c2_mixtral | c3_qwen3next | c4_glm45")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget of the oracle timing leg")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--ffn-rows-per-expert", type=int, default=0,
                    help="FFN-only sweep point: balanced routing with this many rows per expert "
                         "(prefill-shaped batch) on the config's layer shape; reports TFLOP/s")
    ap.add_argument("--placement", default="prefix",
                    help="c5_stream only: how each layer is split between HBM and pinned host memory: "
                         "prefix (the config's block fraction) | hbm | balanced (measured "
                         "beta_cpu / (beta_gpu + beta_cpu), whole down tensors) | budget (--host-budget as "
                         "whole down tensors in every layer) | whole_layer (the last layers entirely on the "
                         "host, same budget) | balanced_raw, budget_raw (the same splits with the host tensors "
                         "stored as dense BF16 and copied, not decoded) | all (the first five)")
    ap.add_argument("--small", action="store_true",
                    help="c5_stream only: a reduced copy of the config (quick functional run, not a result)")
    ap.add_argument("--host-budget", type=float, default=0.125,
                    help="host share of the routed-expert weights for --placement budget / whole_layer")
    ap.add_argument("--exp3", action="store_true",
                    help="standalone decompression in the paper's Exp#3 setting: one GPU's rank-local "
                         "shard of one layer per run, latency mean/std/P99 over repetitions")
    ap.add_argument("--mfma-probe", action="store_true",
                    help="context for the MFMA roofline: rate of a loop of independent BF16 MFMAs with no memory "
                         "traffic, on constant and on random operands (the chip's clock depends on operand content)")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="with --ffn-rows-per-expert: also time torch.matmul (the vendor BLAS) on the two GEMM shapes "
                         "with B stored [K][N] as the slots hold it (context, not part of the path)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain 1 GiB device copies (known traffic) and report their rate; "
                         "under rocprofv3 --pmc they calibrate FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); "
                 "run with --gpus 1")

    import numpy as np
    import torch
    from paper_2604_02715_amd import binding as B
    from paper_2604_02715_amd import harness, inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.mfma_probe:
        return bench_mfma_probe(args)
    if args.exp3:
        return bench_exp3(args)
    cfg = inputs.CONFIGS[args.config]
    if cfg.n_layers > 1:
        if args.small:
            cfg = inputs.scaled(cfg, name=cfg.name + "_small", n_experts=16, hidden=512, ffn=768, tokens=64,
                                top_k=4, n_slots=12, n_layers=6)
        return bench_streaming(cfg, args)
    if args.ffn_rows_per_expert:
        return bench_ffn_rows(cfg, args)
    t_setup = time.time()
    pool = harness.ExpertPool(cfg)
    w13, w2 = harness.make_layer_on_host(cfg, 0, 0, gen_device="cuda")
    blob = pool.encode_layer(0, w13, w2)
    pool.bind_layer(0, blob)
    info = B.fluxmoe_layer_info_get(pool.ctx, 0)
    x = inputs.activations(cfg).cuda()
    ids_np, g_np = inputs.routing(cfg)
    ids, g = torch.from_numpy(ids_np).cuda(), torch.from_numpy(g_np).cuda()
    out = torch.zeros((cfg.tokens, cfg.hidden), dtype=torch.float32, device="cuda")
    union = inputs.routed_union(ids_np)
    # a routed union larger than the slot budget is served in waves (materialize, FFN over the mapped
    # experts accumulating into out, release), as the forward proxy of Sec. 3 does
    n_slots = cfg.n_slots
    waves = [union[i:i + n_slots] for i in range(0, len(union), n_slots)]
    perm = inputs.slot_permutation(n_slots, cfg.name, "bench")
    n_fit = len(union)
    pool.reset_page_table()
    setup_s = time.time() - t_setup

    def step():
        for wi, w in enumerate(waves):
            pool.materialize(0, w, perm[:len(w)])
            flags = (B.FFN_SKIP_UNMAPPED if len(waves) > 1 else 0) | (B.FFN_ACCUMULATE if wi else 0)
            pool.expert_ffn(0, x, ids, g, out, flags)
            if len(waves) > 1:
                pool.release(0, w)

    # bytes one step moves / computes
    dense_bytes = int(n_fit) * (cfg.sigma1 + cfg.sigma2)
    comp_blocks = 0
    for e in union:
        for d in (1, 2):
            comp_blocks += B.fluxmoe_tensor_blocks(pool.ctx, 0, d, int(e))[1]
    comp_bytes = comp_blocks * 4096
    pairs = int(ids_np.size)
    flops = 6.0 * cfg.hidden * cfg.ffn * pairs

    if not args.no_check:
        step()
        torch.cuda.synchronize()
        assert pool.device_errors() == 0
        for e, s in zip(waves[-1], perm):                     # the last wave's experts are still in their slots
            ref = w13[int(e)].reshape(-1).view(torch.int16).cuda()
            assert torch.equal(pool.slot13(int(s)), ref), "decode mismatch"
            ref = w2[int(e)].reshape(-1).view(torch.int16).cuda()
            assert torch.equal(pool.slot2(int(s)), ref), "decode mismatch"
        del ref

    copy_gbps = None
    if args.copy_calibration:
        # 1 GiB device copies of known traffic (1 GiB read + 1 GiB written each): the library's
        # streaming copy (same 16-byte non-temporal accesses as the decode kernel) and torch's
        n = 1 << 30
        src = torch.arange(n // 4, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        copy_gbps = {}
        for name, fn in (("fluxmoe_stream_copy", lambda: B.fluxmoe_stream_copy(
                              dst.data_ptr(), src.data_ptr(), n, 262144, torch.cuda.current_stream().cuda_stream)),
                         ("torch_copy", lambda: dst.copy_(src))):
            fn()
            torch.cuda.synchronize()
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ev0.record()
            for _ in range(5):
                fn()
            ev1.record()
            torch.cuda.synchronize()
            copy_gbps[name] = round(5 * 2 * n / (ev0.elapsed_time(ev1) * 1e-3) / 1e9, 1)
        assert torch.equal(src, dst)
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # timed region: only the decode kernel (the roofline's kernel) is bracketed by events; an event
    # between two kernels idles the device for a few microseconds
    B.fluxmoe_profile_enable(pool.ctx, True, only_kinds=("decode",))
    B.fluxmoe_profile_collect(pool.ctx)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = B.fluxmoe_profile_collect(pool.ctx)
    # per-kernel breakdown of the FFN: a few more steps, untimed, every kernel bracketed
    n_break = max(1, min(args.steps, 5))
    B.fluxmoe_profile_enable(pool.ctx, True)
    for _ in range(n_break):
        step()
    torch.cuda.synchronize()
    prof_ffn = B.fluxmoe_profile_collect(pool.ctx)
    B.fluxmoe_profile_enable(pool.ctx, False)
    assert pool.device_errors() == 0
    for k in ("grouping", "gemm1_swiglu", "gemm2", "combine"):
        prof[k] = prof_ffn[k]

    ms_per_step = elapsed / args.steps * 1e3
    n_launch = len(waves)                                    # decode launches per step
    pattern_probe = access_pattern_probe(comp_blocks // n_launch, dense_bytes / comp_blocks)
    decode_ms = prof["decode"][0] / max(1, prof["decode"][1])            # mean launch
    decode_step_ms = decode_ms * n_launch
    ffn_ms = sum(prof[k][0] for k in ("grouping", "gemm1_swiglu", "gemm2", "combine")) / n_break
    achieved = (comp_bytes + dense_bytes) / (decode_step_ms * 1e-3) / 1e9

    # HBM bytes per launch from hardware counters (two rocprofv3 --pmc runs, summarised in profiles/): only
    # valid for the kernel source they were measured on, so the record carries a hash of that source and a
    # record taken on another version of the kernel is not reported
    traffic, traffic_note = None, None
    tpath = os.path.join(ROOT, "profiles", "decode_traffic.json")
    if os.path.exists(tpath):
        rec = json.load(open(tpath))
        if rec.get("kernel_source_sha256") != decode_kernel_source_hash():
            traffic_note = "profiles/decode_traffic.json was measured on another version of the decode kernel"
        elif cfg.name in rec.get("workloads", {}):
            traffic = rec["workloads"][cfg.name].get("hbm_bytes_per_launch")

    result = {
        "metric": "expert_materialization_dense_out",
        "value": round(dense_bytes / (ms_per_step * 1e-3) / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": cfg.name, "experts": cfg.n_experts, "hidden": cfg.hidden, "ffn": cfg.ffn,
                   "tokens": cfg.tokens, "top_k": cfg.top_k, "experts_materialized_per_step": int(n_fit),
                   "waves_per_step": len(waves), "block_bytes": 4096,
                   "step": "materialize + expert FFN on one stream" + (" per wave of n_slots experts, then release" if len(waves) > 1 else "")},
        "roofline": {"kernel": "decode_kernel", "bound": "hbm", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": traffic, **({"traffic_note": traffic_note} if traffic_note else {}),
                     "algorithmic_bytes_per_launch": (comp_bytes + dense_bytes) // n_launch,
                     "launches_per_step": n_launch, "avg_launch_ms": round(decode_ms, 4)},
        "materialize": {"dense_out_GBps": round(dense_bytes / (decode_step_ms * 1e-3) / 1e9, 1),
                        "compressed_bytes": comp_bytes, "dense_bytes": dense_bytes,
                        "compressed_over_dense": round(comp_bytes / dense_bytes, 4),
                        "payload_saving": round(1 - (8 + (info.payload_bits[0] + info.payload_bits[1]) /
                                                     (info.elements[0] + info.elements[1])) / 16, 4)},
        "ffn": {"TFLOPs": round(flops / (ffn_ms * 1e-3) / 1e12, 2), "ms": round(ffn_ms, 4),
                "frac_mfma_peak": round(flops / (ffn_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                "weight_stream_GBps": round(dense_bytes / (ffn_ms * 1e-3) / 1e9, 1),
                "frac_hbm_peak": round(dense_bytes / (ffn_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "pairs": pairs,
                "kernels_ms": {k: round(prof[k][0] / max(1, prof[k][1]), 4)
                               for k in ("grouping", "gemm1_swiglu", "gemm2", "combine")}},
        "setup_s": round(setup_s, 1),
    }
    if copy_gbps is not None:
        result["device_copy_GBps"] = copy_gbps                # read + write bytes of plain copies
    if pattern_probe is not None:
        pattern_probe["decode_over_probe"] = round(achieved / pattern_probe["GBps"], 4)
        result["decode_access_pattern_probe"] = pattern_probe

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(pool, cfg, blob, w13, w2, args.cpu_seconds)
        try:
            result["cpu_baseline"]["expert_ffn"] = cpu_baseline_ffn(cfg, x.cpu(), ids_np, g_np, w13, w2)
        except Exception as exc:                                  # the decode figure stands on its own
            result["cpu_baseline"]["expert_ffn"] = {"error": str(exc)[:200]}
    print(json.dumps(result), flush=True)
    pool.close()


def access_pattern_probe(n_blocks, out_bytes_per_block, reps=5):
    """What HBM gives the decode kernel's access pattern on this machine: a kernel of the same launch shape that
    reads n_blocks blocks of 4 KiB, one per wavefront, and writes out_bytes_per_block (on average) for each in
    1 KiB pieces, with nothing in between (fluxmoe_stream_mix).  Untimed leg, after the timed steps."""
    import torch
    from paper_2604_02715_amd import binding as B
    small = max(128, int(round((out_bytes_per_block - 48) / 128.0)) * 128)   # three blocks of eight write 128 more
    waves = int(os.environ.get("FLUXMOE_DECODE_WAVES", "8"))
    per_wave = int(os.environ.get("FLUXMOE_DECODE_BLOCKS_PER_WAVE", "3"))
    if n_blocks < 1 or waves not in (4, 8, 16) or not 1 <= per_wave <= 1024:
        return None
    src = torch.empty(n_blocks * 4096, dtype=torch.uint8, device="cuda").random_(0, 256)
    dst = torch.empty(n_blocks * (small + 128), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    run = lambda: B.fluxmoe_stream_mix(dst.data_ptr(), dst.numel(), src.data_ptr(), src.numel(), small, waves,
                                       per_wave, 0, stream)
    written = run()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(reps):
        run()
    ev1.record()
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / reps
    return {"GBps": round((src.numel() + written) / (ms * 1e-3) / 1e9, 1), "ms": round(ms, 4),
            "bytes_read": src.numel(), "bytes_written": written,
            "what": "fluxmoe_stream_mix: the decode launch's shape, loads and stores without the decoding"}


def decode_kernel_source_hash():
    """sha256 over the sources the decode kernel is compiled from."""
    import hashlib
    h = hashlib.sha256()
    for name in ("decode_kernel.hip", "decode_args.h"):
        h.update(open(os.path.join(ROOT, "paper_2604_02715_amd", "csrc", name), "rb").read())
    return h.hexdigest()


def bench_exp3(args):
    """Exp#3 of the paper (Sec. 6.3, Tab. 'standalone_decompression'): each run decodes the
    routed-expert shard of one layer that one GPU of the paper's deployment holds (expert
    parallel: Mixtral 8/2 = 4 experts, Qwen3-Next 512/4 = 128, GLM-4.5 160/8 = 20); throughput =
    uncompressed BF16 volume / decode time.  The two tensor types are issued on two streams
    (fluxmoe_materialize_two_streams) as the paper's loading path does (Sec. 5), and a layer's latency runs
    from issue until both types are ready; the one-launch figure (both types in one kernel, what
    fluxmoe_materialize does) is reported beside it.  The paper's numbers (L40S / H20) are context only;
    its Mixtral shard is the 87.5 % GPU-tier share (1.23 GB), here the 4 whole experts (1.41 GB)."""
    import numpy as np
    import torch
    from paper_2604_02715_amd import binding as B
    from paper_2604_02715_amd import harness, inputs

    paper = {"c2_mixtral": (4, "1x L40S", 1.23, 3.07, 3.13, 401.9),
             "c3_qwen3next": (128, "1x L40S", 0.81, 2.03, 2.07, 396.5),
             "c4_glm45": (20, "1x H20", 0.94, 2.17, 2.17, 435.4)}
    reps = max(args.steps, 30)
    rows = []
    for name, (n_exp, hw, p_gb, p_avg, p_p99, p_tp) in paper.items():
        cfg = inputs.scaled(inputs.CONFIGS[name], n_experts=n_exp, n_slots=n_exp)
        pool = harness.ExpertPool(cfg)
        w13, w2 = harness.make_layer_on_host(cfg, 0, 0, gen_device="cuda")
        pool.bind_layer(0, pool.encode_layer(0, w13, w2))
        pool.reset_page_table()
        ids = np.arange(n_exp)
        slots = inputs.slot_permutation(n_exp, name, "exp3")
        pool.materialize(0, ids, slots)
        torch.cuda.synchronize()
        for e, s_ in zip(ids[:2], slots[:2]):
            assert torch.equal(pool.slot13(int(s_)), w13[int(e)].reshape(-1).view(torch.int16).cuda())
        lat1 = []
        for _ in range(reps):
            B.fluxmoe_profile_enable(pool.ctx, True)
            B.fluxmoe_profile_collect(pool.ctx)
            pool.materialize(0, ids, slots)
            torch.cuda.synchronize()
            lat1.append(B.fluxmoe_profile_collect(pool.ctx)["decode"][0])
        B.fluxmoe_profile_enable(pool.ctx, False)
        # two streams, issue -> both types ready: events on the first stream around the call (it joins the second)
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        lat = []
        for _ in range(reps + 3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(s1)
            pool.materialize_two_streams(0, ids, slots, s1, s2)
            e1.record(s1)
            torch.cuda.synchronize()
            lat.append(e0.elapsed_time(e1))
        lat = np.asarray(lat[3:])
        for e, s_ in zip(ids[-2:], slots[-2:]):
            assert torch.equal(pool.slot2(int(s_)), w2[int(e)].reshape(-1).view(torch.int16).cuda())
        assert pool.device_errors() == 0
        lat1 = np.asarray(lat1)
        dense = n_exp * (cfg.sigma1 + cfg.sigma2)
        comp = sum(B.fluxmoe_tensor_blocks(pool.ctx, 0, d, e)[1] for e in range(n_exp) for d in (1, 2)) * 4096
        tp = dense / (lat * 1e-3) / 1e9
        rows.append({"model_shape": name, "experts_per_gpu": n_exp, "dense_GB": round(dense / 1e9, 3),
                     "storage_saved_incl_framing": round(1 - comp / dense, 4),
                     "latency_ms_mean": round(float(lat.mean()), 4), "latency_ms_std": round(float(lat.std()), 4),
                     "latency_ms_p99": round(float(np.percentile(lat, 99)), 4),
                     "throughput_GBps_mean": round(float(tp.mean()), 1), "throughput_GBps_std": round(float(tp.std()), 1),
                     "frac_hbm_peak": round(float(((comp + dense) / (lat * 1e-3) / 1e9).mean()) / HBM_PEAK_GBPS, 4),
                     "one_launch_latency_ms_mean": round(float(lat1.mean()), 4),
                     "one_launch_throughput_GBps_mean": round(float((dense / (lat1 * 1e-3) / 1e9).mean()), 1),
                     "paper_context": {"hardware": hw, "dense_GB": p_gb, "latency_ms": p_avg, "p99_ms": p_p99,
                                       "throughput_GBps": p_tp}})
        pool.close()
        del w13, w2
    print(json.dumps({"metric": "standalone_decompression_exp3", "unit": "GB/s", "n_gpus": 1, "steps": reps,
                      "value": rows[0]["throughput_GBps_mean"], "dtype": "bf16", "data": "synthetic",
                      "vs_baseline": None, "higher_is_better": True, "rows": rows}), flush=True)


def bench_mfma_probe(args):
    """MFMA-only loop (fluxmoe_mfma_probe) on three operand contents."""
    import numpy as np
    import torch
    from paper_2604_02715_amd import binding as B

    n_wg, iters = torch.cuda.get_device_properties(0).multi_processor_count, 200000
    out = torch.zeros(n_wg * 256, dtype=torch.float32, device="cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    contents = {
        "constant": torch.full((32768,), 1.0, dtype=torch.bfloat16, device="cuda"),
        "gaussian": torch.randn(32768, generator=g, device="cuda").to(torch.bfloat16),
        "random_bits": (torch.randint(0, 1 << 16, (32768,), generator=g, device="cuda", dtype=torch.int32) & 0xBFFF
                        ).to(torch.int16).view(torch.bfloat16),      # any sign/mantissa, exponent below 2^64
    }
    res = {}
    for name, t in contents.items():
        best = None
        for _ in range(3):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            B.fluxmoe_mfma_probe(t.data_ptr(), out.data_ptr(), n_wg, iters, torch.cuda.current_stream().cuda_stream)
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b)
            best = ms if best is None else min(best, ms)
        flops = n_wg * 4.0 * iters * 16 * 32768
        res[name] = {"ms": round(best, 3), "TFLOPs": round(flops / (best * 1e-3) / 1e12, 1),
                     "frac_of_peak": round(flops / (best * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
    print(json.dumps({"metric": "mfma_only_loop", "unit": "TFLOP/s", "n_gpus": 1, "dtype": "bf16",
                      "config": {"workload": "mfma_probe", "workgroups": n_wg, "iters": iters,
                                 "mfma": "v_mfma_f32_32x32x16_bf16, 16 accumulators per wavefront, 4 wavefronts per CU"},
                      "peak": MFMA_BF16_PEAK_TFLOPS, "operands": res}), flush=True)


def bench_ffn_rows(cfg, args):
    """FFN only, M rows per expert on every expert of the layer (balanced synthetic routing):
    the MFMA-bound side of the expert GEMM.  Materialization runs once, untimed."""
    import numpy as np
    import torch
    from paper_2604_02715_amd import binding as B
    from paper_2604_02715_amd import harness, inputs

    M, E, K = args.ffn_rows_per_expert, cfg.n_experts, cfg.top_k
    T = M * E // K
    big = inputs.scaled(cfg, tokens=T)
    pool = harness.ExpertPool(big)
    w13, w2 = harness.make_layer_on_host(cfg, 0, 0, gen_device="cuda")
    pool.bind_layer(0, pool.encode_layer(0, w13, w2))
    pool.reset_page_table()
    pool.materialize(0, np.arange(E), np.arange(E))
    t = np.arange(T)
    ids_np = np.stack([(t + j * (E // K)) % E for j in range(K)], axis=1).astype(np.int32)
    assert (np.bincount(ids_np.reshape(-1), minlength=E) == M).all()
    g_np = np.full((T, K), 1.0 / K, dtype=np.float32)
    x = inputs.activations(big).cuda()
    ids, g = torch.from_numpy(ids_np).cuda(), torch.from_numpy(g_np).cuda()
    out = torch.zeros((T, cfg.hidden), dtype=torch.float32, device="cuda")
    for _ in range(max(1, args.warmup)):
        pool.expert_ffn(0, x, ids, g, out)
    torch.cuda.synchronize()
    B.fluxmoe_profile_enable(pool.ctx, True)
    B.fluxmoe_profile_collect(pool.ctx)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        pool.expert_ffn(0, x, ids, g, out)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    prof = B.fluxmoe_profile_collect(pool.ctx)
    assert pool.device_errors() == 0
    flops = 6.0 * cfg.hidden * cfg.ffn * T * K
    g1 = prof["gemm1_swiglu"][0] / args.steps
    g2 = prof["gemm2"][0] / args.steps
    # spot check against the oracle on two tokens
    if not args.no_check:
        from oracle import ffn as offn
        sel = np.array([0, T - 1])
        want = offn.moe_ffn(inputs.bits_u16(x.cpu())[sel], ids_np[sel], g_np[sel],
                            lambda e: (inputs.bits_u16(w13[e]), inputs.bits_u16(w2[e])), round_h=True)
        err = offn.rel_frobenius(out[torch.from_numpy(sel).cuda()].cpu().numpy(), want)
        assert err <= 1e-3, err
    tf = flops / (ms * 1e-3) / 1e12
    vendor = None
    if args.vendor_gemm:
        # one [rows][K] x [K][N] product per GEMM shape with all T*K rows against one expert's matrix:
        # the same flops as the grouped product
        def mm(rows, kk, nn):
            aa = torch.randn(rows, kk, device="cuda").to(torch.bfloat16)
            bb = (torch.randn(kk, nn, device="cuda") * 0.02).to(torch.bfloat16)
            for _ in range(3):
                aa @ bb
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                aa @ bb
            e1.record()
            torch.cuda.synchronize()
            return 2.0 * rows * kk * nn / (e0.elapsed_time(e1) / 10 * 1e-3) / 1e12
        vendor = {"what": "torch.matmul bf16, B row-major [K][N], one product of all rows per GEMM shape",
                  "gemm1_TFLOPs": round(mm(T * K, cfg.hidden, 2 * cfg.ffn), 1),
                  "gemm2_TFLOPs": round(mm(T * K, cfg.ffn, cfg.hidden), 1)}
    print(json.dumps({
        "metric": "expert_ffn_throughput", "value": round(tf, 1), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name + "_ffn_rows", "rows_per_expert": M, "experts": E, "hidden": cfg.hidden,
                   "ffn": cfg.ffn, "tokens": T, "top_k": K},
        # below the ridge (2.5 PFLOP/s / 8 TB/s = 312 rows per expert) streaming the weights once bounds the
        # kernel, above it the matrix cores do
        "roofline": ({"kernel": "gemm1_swiglu", "bound": "mfma",
                      "achieved": round(4.0 * cfg.hidden * cfg.ffn * T * K / (g1 * 1e-3) / 1e12, 1),
                      "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                      "frac": round(4.0 * cfg.hidden * cfg.ffn * T * K / (g1 * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                      "traffic": None, "avg_launch_ms": round(g1, 4)} if M >= 312 else
                     {"kernel": "gemm1_swiglu", "bound": "hbm",
                      "achieved": round(E * cfg.sigma1 / (g1 * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                      "frac": round(E * cfg.sigma1 / (g1 * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                      "traffic": None, "algorithmic_bytes_per_launch": E * cfg.sigma1, "avg_launch_ms": round(g1, 4)}),
        "ffn": {"frac_mfma_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                "gemm2_TFLOPs": round(2.0 * cfg.hidden * cfg.ffn * T * K / (g2 * 1e-3) / 1e12, 1),
                "kernels_ms": {k: round(prof[k][0] / max(1, prof[k][1]), 4)
                               for k in ("grouping", "gemm1_swiglu", "gemm2", "combine")}},
        "vendor_gemm": vendor}), flush=True)
    pool.close()


def bench_streaming(cfg, args):
    """Config 5: all layers in order through two slot halves, part of every layer's compressed
    blocks in pinned host memory fetched on a side stream; steady-state time per layer.
    --placement selects the tier split (Sec. 4.2 "Memory hierarchy model" and the whole-layer
    ablation of Sec. 6.1)."""
    import math

    import numpy as np
    import torch
    from paper_2604_02715_amd import binding as B
    from paper_2604_02715_amd import harness, inputs

    t0 = time.time()
    placements = (["hbm", "balanced", "budget", "whole_layer", "prefix"] if args.placement == "all"
                  else args.placement.split(","))
    pool = harness.ExpertPool(cfg)
    blobs = {}
    for layer in range(cfg.n_layers):
        w13, w2 = harness.make_layer_on_host(cfg, layer, 0, gen_device="cuda")
        blob = pool.encode_layer(layer, w13, w2)
        blobs[layer] = blob.clone()
        del w13, w2, blob
        print("layer %d encoded (%.0f s)" % (layer, time.time() - t0), file=sys.stderr, flush=True)
    routings = [inputs.routing(cfg, layer) for layer in range(cfg.n_layers)]
    xs = [inputs.activations(cfg, layer).cuda() for layer in range(cfg.n_layers)]
    outs = [torch.zeros((cfg.tokens, cfg.hidden), dtype=torch.float32, device="cuda") for _ in xs]
    dense_layer = cfg.n_experts * (cfg.sigma1 + cfg.sigma2)
    E = cfg.n_experts

    def measure_betas():
        """beta_gpu: dense BF16 bytes per second of decoding HBM-resident blocks; beta_cpu: the
        same for host-tier blocks, i.e. the pinned-host DMA rate divided by the pool's
        compressed/dense ratio."""
        pool.bind_layer(0, blobs[0], 0.0, check=False)
        pool.reset_page_table()
        half = cfg.n_slots // 2
        ids = list(range(half))
        B.fluxmoe_profile_enable(pool.ctx, True)
        for i in range(6):
            if i == 1:
                torch.cuda.synchronize()
                B.fluxmoe_profile_collect(pool.ctx)
            pool.materialize(0, ids, ids)
        torch.cuda.synchronize()
        ms, n = B.fluxmoe_profile_collect(pool.ctx)["decode"]
        B.fluxmoe_profile_enable(pool.ctx, False)
        beta_gpu = half * (cfg.sigma1 + cfg.sigma2) / (ms / n * 1e-3)
        nbytes = min(1 << 29, blobs[0].numel())
        src = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
        src.copy_(blobs[0][:nbytes])
        dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        dst.copy_(src, non_blocking=True)
        a.record()
        for _ in range(3):
            dst.copy_(src, non_blocking=True)
        b.record()
        torch.cuda.synchronize()
        pcie = 3 * nbytes / (a.elapsed_time(b) * 1e-3)
        ratio = pool.blob_bytes[0] / dense_layer
        del src, dst
        return beta_gpu, pcie / ratio, pcie

    def host_tensors_of(n_down, n_fused):
        """Largest expert indices first (the planner's order, Sec. 4.3)."""
        return [(2, e) for e in range(E - n_down, E)] + [(1, e) for e in range(E - n_fused, E)]

    streams = None
    for placement in placements:
        t1 = time.time()
        pool.host_blobs.clear()
        pool.tensor_copies.clear()
        torch.cuda.synchronize()
        if hasattr(torch._C, "_host_emptyCache"):
            torch._C._host_emptyCache()                      # give pinned buffers of the last placement back
        info = {"placement": placement}
        if placement.endswith("_raw"):
            info["host_tier_format"] = "dense BF16 (share below is dense host bytes over the compressed pool)"
        host_bytes = []
        raw = placement.endswith("_raw")                     # host tensors stored dense (tier 2), not compressed
        if placement in ("balanced", "balanced_raw"):
            beta_gpu, beta_cpu, pcie = measure_betas()
            if raw:
                beta_cpu = pcie                              # dense bytes cross PCIe as they are
            x_bw, n_down, n_fused = B.fluxmoe_balanced_split(beta_gpu, beta_cpu, E)
            info.update(beta_gpu_GBps=round(beta_gpu / 1e9, 1), beta_cpu_GBps=round(beta_cpu / 1e9, 1),
                        pcie_GBps=round(pcie / 1e9, 1), x_bw=round(x_bw, 5), host_down_tensors=n_down,
                        host_fused_tensors=n_fused, x_realised=round((n_down + 2 * n_fused) / (3 * E), 5))
        elif placement in ("budget", "budget_raw"):
            units = math.ceil(3 * E * args.host_budget - 1e-12)
            n_down = min(units, E)
            n_fused = min(E, (units - n_down + 1) // 2)
            info.update(host_budget=args.host_budget, host_down_tensors=n_down, host_fused_tensors=n_fused,
                        x_realised=round((n_down + 2 * n_fused) / (3 * E), 5))
        n_host_layers = math.ceil(args.host_budget * cfg.n_layers - 1e-12) if placement == "whole_layer" else 0
        for layer in range(cfg.n_layers):
            frac = {"prefix": cfg.host_fraction, "whole_layer": 1.0 if layer >= cfg.n_layers - n_host_layers else 0.0}.get(placement, 0.0)
            _, n_host = pool.bind_layer(layer, blobs[layer], frac, check=(layer == 0))
            hb = n_host * 4096
            if placement in ("balanced", "budget"):
                hb = pool.place_tensors_on_host(layer, blobs[layer], host_tensors_of(n_down, n_fused))
            elif raw:
                w13, w2 = inputs.layer_weights(cfg, layer, device="cuda")
                hb = pool.place_tensors_raw_on_host(
                    layer, [((t, e), (w2[e] if t == 2 else w13[e]).cpu()) for (t, e) in host_tensors_of(n_down, n_fused)])
                del w13, w2
            host_bytes.append(hb)
        if placement == "whole_layer":
            info.update(host_budget=args.host_budget, host_layers=n_host_layers)
        if max(host_bytes) > 0:
            pool.bind_staging(2 * max(host_bytes) + 8192)
        proxy = harness.StreamingProxy(pool, routings, xs, outs, streams=streams)
        streams = (proxy.load_stream, proxy.infer_stream, proxy.copy_stream)
        pool.reset_page_table()
        setup_s = time.time() - t1
        print("placement %s bound (%.0f s)" % (placement, setup_s), file=sys.stderr, flush=True)

        # parity on the fly: one overlapped pass, then the slots of the last two layers' last waves
        # still hold their experts; compare them with regenerated originals
        proxy.run_pass()
        torch.cuda.synchronize()
        assert pool.device_errors() == 0
        if not args.no_check:
            for layer in (cfg.n_layers - 2, cfg.n_layers - 1):
                w13, w2 = inputs.layer_weights(cfg, layer, device="cuda")
                w, slots = proxy.plan[layer][1][-1]
                for e, s_ in zip(w, slots):
                    assert torch.equal(pool.slot13(int(s_)), w13[int(e)].reshape(-1).view(torch.int16)), "decode mismatch"
                    assert torch.equal(pool.slot2(int(s_)), w2[int(e)].reshape(-1).view(torch.int16)), "decode mismatch"
                del w13, w2

        def timed_passes(n_pass, **kw):
            per_layer, whole = [], []
            for _ in range(n_pass):
                evs = [torch.cuda.Event(enable_timing=True) for _ in range(cfg.n_layers)]
                start = torch.cuda.Event(enable_timing=True)
                start.record(proxy.infer_stream)
                proxy.run_pass(layer_done_events=evs, **kw)
                torch.cuda.synchronize()
                per_layer.append([evs[i - 1].elapsed_time(evs[i]) for i in range(1, cfg.n_layers)])
                whole.append(start.elapsed_time(evs[-1]))
            return np.asarray(per_layer), np.asarray(whole)

        for _ in range(args.warmup if args.warmup < 3 else 1):
            proxy.run_pass()
        torch.cuda.synchronize()
        n_pass = max(1, min(args.steps, 5))
        t2 = time.perf_counter()
        pl, whole = timed_passes(n_pass)
        wall = time.perf_counter() - t2
        steady = pl[:, 1:]                                   # layers 2..N-1 of every pass
        per_layer_ms = float(steady.mean())

        # isolated components per layer: host fetch (layer with the most host bytes), decode, FFN
        B.fluxmoe_profile_enable(pool.ctx, True)
        B.fluxmoe_profile_collect(pool.ctx)
        proxy.run_pass(single_stream=True)
        torch.cuda.synchronize()
        prof = B.fluxmoe_profile_collect(pool.ctx)
        B.fluxmoe_profile_enable(pool.ctx, False)
        decode_ms = prof["decode"][0] / cfg.n_layers
        ffn_ms = sum(prof[k][0] for k in ("grouping", "gemm1_swiglu", "gemm2", "combine")) / cfg.n_layers
        copy_ms, pcie_rate = 0.0, None
        if max(host_bytes) > 0:
            hl = int(np.argmax(host_bytes))
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ev0.record(proxy.copy_stream)
            pool.prefetch_host(hl, proxy.plan[hl][0], proxy.copy_stream)
            ev1.record(proxy.copy_stream)
            torch.cuda.synchronize()
            copy_ms = ev0.elapsed_time(ev1)
            if placement in ("prefix", "whole_layer"):
                fetched = host_bytes[hl] * len(proxy.plan[hl][0]) / E
            else:
                routed = set(int(v) for v in proxy.plan[hl][0])
                fetched = sum((cfg.sigma2 if t == 2 else cfg.sigma1) if raw else B.fluxmoe_tensor_blocks(pool.ctx, hl, t, e)[1] * 4096
                              for (t, e) in host_tensors_of(n_down, n_fused) if e in routed)
            pcie_rate = round(fetched / (copy_ms * 1e-3) / 1e9, 1)
        union = np.mean([len(u) for u, _ in proxy.plan])
        dense_bytes = union * (cfg.sigma1 + cfg.sigma2)
        result = {
            "metric": "streaming_steady_state_per_layer", "value": round(per_layer_ms, 3), "unit": "ms",
            "n_gpus": 1, "steps": n_pass, "warmup": 1, "ms_per_step": round(wall / n_pass * 1e3, 2),
            "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": cfg.name, "layers": cfg.n_layers, "experts": cfg.n_experts, "hidden": cfg.hidden,
                       "ffn": cfg.ffn, "tokens": cfg.tokens, "top_k": cfg.top_k, "slots": cfg.n_slots,
                       "host_share_of_pool": round(sum(host_bytes) / sum(pool.blob_bytes.values()), 4),
                       "mean_routed_union": round(float(union), 1),
                       "waves_per_layer": round(float(np.mean([len(w) for _, w in proxy.plan])), 2), **info},
            "per_layer": {"steady_ms_mean": round(per_layer_ms, 3), "steady_ms_std": round(float(steady.std()), 3),
                          "steady_ms_max": round(float(steady.max()), 3),
                          "pass_ms_over_layers": round(float(whole.mean()) / cfg.n_layers, 3),
                          "host_fetch_ms_isolated": round(copy_ms, 3), "decode_ms_isolated": round(decode_ms, 3),
                          "ffn_ms_isolated": round(ffn_ms, 3), "pcie_GBps": pcie_rate,
                          # the longer of the two isolated legs over the measured steady-state time: 1.0 means the
                          # per-layer time equals its longest leg (the other one is fully hidden behind it); with no
                          # host tier the longest leg is decode + FFN back to back, so the ratio says nothing about overlap
                          "longest_leg_over_measured": (round(max(copy_ms, decode_ms + ffn_ms) / per_layer_ms, 3)
                                                        if placement != "whole_layer" else None),
                          "dense_out_GBps": round(dense_bytes / (per_layer_ms * 1e-3) / 1e9, 1)},
            "setup_s": round(setup_s + (t1 - t0 if placement == placements[0] else 0), 1),
        }
        print(json.dumps(result), flush=True)
        del proxy
    pool.close()


def cpu_baseline(pool, cfg, blob, w13, w2, budget_s):
    """The oracle decoder, as it stands, on a bounded sample of the same pool (rank 0, host):
    whole tensors in blob order (down tensors of experts 0, 1, ...) until the time budget."""
    import numpy as np
    from oracle import codec
    from paper_2604_02715_amd import binding as B
    from paper_2604_02715_amd import inputs

    blocks = blob.numpy().reshape(-1, 4096)
    elems, n_blocks_done, tensors = 0, 0, 0
    t0 = time.perf_counter()
    for d, arr in ((2, w2), (1, w13)):
        lens = B.fluxmoe_code_lengths(pool.ctx, 0, d)
        for e in range(cfg.n_experts):
            if time.perf_counter() - t0 >= budget_s:
                break
            b0, nb = B.fluxmoe_tensor_blocks(pool.ctx, 0, d, e)
            want = inputs.bits_u16(arr[e]).reshape(-1)
            got = codec.decode_tensor(blocks[b0:b0 + nb], lens, want.size, chunk=256)
            assert np.array_equal(got, want), "oracle decode mismatch"
            elems += want.size
            n_blocks_done += nb
            tensors += 1
    dt = time.perf_counter() - t0
    res = {"value": round(2.0 * elems / dt / 1e9, 5), "unit": "GB/s", "cores": 1, "kind": "oracle",
           "sample": "oracle/codec.decode_tensor on the first %d tensors of this pool in blob order "
                     "(%d blocks, %d elements, %.1f s, numpy, one thread)" % (tensors, n_blocks_done, elems, dt)}
    try:
        res["all_cores"] = cpu_baseline_all_cores(pool, cfg, blocks, w2, max(1, tensors))
    except Exception as exc:                                  # the single-thread figure stands on its own
        res["all_cores"] = {"error": str(exc)[:200]}
    return res


def cpu_baseline_ffn(cfg, x, ids_np, g_np, w13, w2):
    """The FP64 FFN oracle, as it stands (oracle/ffn.moe_ffn, h rounded to BF16), on a bounded sample of the
    same batch: every (token, k) pair routed to the busiest expert, i.e. one expert's whole row group.  Timed
    with one BLAS thread and with all host threads; the time includes the oracle's widening of the expert's
    BF16 weights to FP64.  FLOPs = 6 H F per pair."""
    import numpy as np
    from oracle import ffn as offn
    from paper_2604_02715_amd import inputs
    import threadpoolctl

    counts = np.bincount(ids_np.reshape(-1), minlength=cfg.n_experts)
    e = int(counts.argmax())
    pairs = int(counts[e])
    xb = inputs.bits_u16(x)
    weights = lambda k: (inputs.bits_u16(w13[k]), inputs.bits_u16(w2[k]))
    flops = 6.0 * cfg.hidden * cfg.ffn * pairs
    res = {"unit": "TFLOP/s", "kind": "oracle",
           "sample": "oracle/ffn.moe_ffn (FP64, h rounded to BF16) on the %d pairs routed to expert %d of this batch, "
                     "%.2f GFLOP, weight widening included" % (pairs, e, flops / 1e9)}
    for label, limit in (("one_thread", 1), ("all_threads", None)):
        with threadpoolctl.threadpool_limits(limits=limit):
            t0 = time.perf_counter()
            out = offn.moe_ffn(xb, ids_np, g_np, weights, round_h=True, mapped={e})
            dt = time.perf_counter() - t0
            threads = 1 if limit == 1 else max(info["num_threads"] for info in threadpoolctl.threadpool_info() or [{"num_threads": os.cpu_count()}])
        assert np.isfinite(out).all()
        res[label] = {"value": round(flops / dt / 1e12, 6), "cores": int(threads), "seconds": round(dt, 2)}
    return res


_WORKER = r'''
import sys, time, numpy as np
sys.path.insert(0, sys.argv[1])
from oracle import codec
d = np.load(sys.argv[2])
blocks, lens, n_elems, want = d["blocks"], d["lens"], int(d["n_elems"]), d["want"]
t_start = float(sys.argv[3])
while time.time() < t_start:
    time.sleep(0.001)
t0 = time.perf_counter()
got = codec.decode_tensor(blocks, lens, n_elems, chunk=256)
dt = time.perf_counter() - t0
assert np.array_equal(got, want), "oracle decode mismatch"
print("%d %.6f %.6f" % (got.size, dt, time.time()))
'''


def cpu_baseline_all_cores(pool, cfg, blocks, w2, per_core_tensors):
    """The same oracle decode on every host core at once: one child process per core (the oracle is
    numpy under the interpreter lock, threads do not scale), each decoding one down tensor of the
    pool (experts round robin); the children import numpy and oracle/ only and start together.
    Throughput = all decoded bytes / (last finish - common start)."""
    import subprocess
    import tempfile
    import numpy as np
    from paper_2604_02715_amd import binding as B
    from paper_2604_02715_amd import inputs

    cores = max(1, min(16, os.cpu_count() or 1))
    lens = np.asarray(B.fluxmoe_code_lengths(pool.ctx, 0, 2))
    with tempfile.TemporaryDirectory(dir="/dev/shm" if os.path.isdir("/dev/shm") else None) as tmp:
        files = []
        for i in range(cores):
            e = i % cfg.n_experts
            b0, nb = B.fluxmoe_tensor_blocks(pool.ctx, 0, 2, e)
            want = inputs.bits_u16(w2[e]).reshape(-1)
            f = os.path.join(tmp, "t%d.npz" % i)
            np.savez(f, blocks=blocks[b0:b0 + nb], lens=lens, n_elems=want.size, want=want)
            files.append(f)
        t_start = time.time() + 4.0                           # interpreter and numpy start-up happen before it
        procs = [subprocess.Popen([sys.executable, "-c", _WORKER, ROOT, f, repr(t_start)],
                                  stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True) for f in files]
        elems, t_end = 0, t_start
        for pr in procs:
            out, err = pr.communicate(timeout=600)
            if pr.returncode != 0:
                raise RuntimeError("oracle worker failed: " + err[-300:])
            n, _, t_fin = out.split()
            elems += int(n)
            t_end = max(t_end, float(t_fin))
    dt = t_end - t_start
    return {"value": round(2.0 * elems / dt / 1e9, 5), "unit": "GB/s", "cores": cores,
            "sample": "one down tensor per core, %d processes started together (%d elements, %.1f s)" % (cores, elems, dt)}


if __name__ == "__main__":
    main()
