"""ctypes binding of libfluxmoe.so: argument marshalling only, same names as include/fluxmoe.h.

Every step of the path runs inside the library's HIP kernels; there is no fallback.  If the
library has not been built, loading raises (build it with python -m paper_2604_02715_amd.build).
Pointers are passed as integers (torch's tensor.data_ptr(), numpy's arr.ctypes.data).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libfluxmoe.so")
_lib = None

FFN_ACCUMULATE = 1
FFN_SKIP_UNMAPPED = 2
TIER_HBM, TIER_HOST, TIER_HOST_RAW = 0, 1, 2

STATUS = {0: "OK", -1: "EINVAL", -2: "ENOMEM", -3: "ECORRUPT", -4: "ERANGE", -5: "EHIP", -6: "ESTATE"}


class FluxmoeError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("fluxmoe %s (%d): %s" % (STATUS.get(status, "?"), status, text))
        self.status = status


class Desc(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("n_layers", "n_experts", "hidden", "ffn", "block_bytes",
                                          "max_code_len", "n_slots", "flags")]


class Sizes(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("sigma1", "sigma2", "slots13_bytes", "slots2_bytes",
                                          "page_table_bytes", "layer_blob_bound",
                                          "pool_workspace_bytes")]


class LayerInfo(C.Structure):
    _fields_ = [("n_blocks", C.c_uint64), ("payload_bits", C.c_uint64 * 2),
                ("elements", C.c_uint64 * 2)]


class PlannerDesc(C.Structure):
    _fields_ = [("n_layers", C.c_uint32), ("experts_per_rank", C.c_uint32),
                ("control_interval", C.c_uint32), ("reserved", C.c_uint32),
                ("theta", C.c_double), ("adjustment_granularity", C.c_double)]


class PlannerMove(C.Structure):
    _fields_ = [("layer", C.c_uint32), ("expert", C.c_uint32), ("type", C.c_int32),
                ("to_host", C.c_int32)]


class PlannerDecision(C.Structure):
    _fields_ = [("action", C.c_int32), ("n_moves", C.c_uint32), ("rho", C.c_double),
                ("tau_eff", C.c_double), ("tau_load", C.c_double)]


class PagedTensorInfo(C.Structure):
    _fields_ = [("granularity", C.c_uint64), ("A", C.c_uint64 * 2), ("S", C.c_uint64 * 2),
                ("v0", C.c_uint64 * 2), ("reusable_window", C.c_uint64 * 2),
                ("virtual_bytes", C.c_uint64), ("physical_bytes", C.c_uint64),
                ("pad_bytes", C.c_uint64), ("n_uncompressed", C.c_uint32), ("n_pageable", C.c_uint32)]


PLAN_KEEP, PLAN_RECLAIM, PLAN_RESTORE, PLAN_SKIP, PLAN_DONE = 0, 1, -1, 2, 3

EXPORTS = {
    "fluxmoe_last_error": (C.c_char_p, []),
    "fluxmoe_create": (C.c_int, [C.POINTER(Desc), C.POINTER(C.c_void_p)]),
    "fluxmoe_destroy": (C.c_int, [C.c_void_p]),
    "fluxmoe_query_sizes": (C.c_int, [C.c_void_p, C.POINTER(Sizes)]),
    "fluxmoe_ffn_workspace_bytes": (C.c_uint64, [C.c_void_p, C.c_uint32, C.c_uint32, C.c_int]),
    "fluxmoe_ffn_plan": (C.c_int, [C.c_void_p, C.c_uint32, C.c_uint32, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]),
    "fluxmoe_encode_pool": (C.c_int, [C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_size_t, C.POINTER(C.c_size_t), C.c_int]),
    "fluxmoe_layer_info_get": (C.c_int, [C.c_void_p, C.c_uint32, C.POINTER(LayerInfo)]),
    "fluxmoe_code_lengths": (C.c_int, [C.c_void_p, C.c_uint32, C.c_int, C.c_void_p]),
    "fluxmoe_tensor_blocks": (C.c_int, [C.c_void_p, C.c_uint32, C.c_int, C.c_uint32,
                                        C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]),
    "fluxmoe_tensor_first_elems": (C.c_int, [C.c_void_p, C.c_uint32, C.c_int, C.c_uint32,
                                             C.c_void_p, C.c_size_t]),
    "fluxmoe_bind_arenas": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t]),
    "fluxmoe_bind_layer": (C.c_int, [C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint64, C.c_void_p,
                                     C.c_void_p]),
    "fluxmoe_set_tensor_backing": (C.c_int, [C.c_void_p, C.c_uint32, C.c_int, C.c_uint32, C.c_int,
                                             C.c_void_p]),
    "fluxmoe_bind_staging": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t]),
    "fluxmoe_reset_page_table": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "fluxmoe_prefetch_host": (C.c_int, [C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32, C.c_void_p]),
    "fluxmoe_materialize": (C.c_int, [C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32, C.c_void_p,
                                      C.c_void_p, C.c_void_p]),
    "fluxmoe_materialize_two_streams": (C.c_int, [C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32, C.c_void_p,
                                                  C.c_void_p, C.c_void_p, C.c_void_p]),
    "fluxmoe_release": (C.c_int, [C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p]),
    "fluxmoe_expert_ffn": (C.c_int, [C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32, C.c_void_p,
                                     C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint32,
                                     C.c_void_p]),
    "fluxmoe_expert_ffn_static": (C.c_int, [C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32, C.c_void_p,
                                            C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint32,
                                            C.c_void_p]),
    "fluxmoe_shared_expert_ffn": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32,
                                            C.c_void_p, C.c_uint32, C.c_void_p]),
    "fluxmoe_stream_copy": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32, C.c_void_p]),
    "fluxmoe_stream_mix": (C.c_int, [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint32,
                                     C.c_uint32, C.c_uint32, C.POINTER(C.c_uint64), C.c_void_p]),
    "fluxmoe_mfma_probe": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p]),
    "fluxmoe_profile_enable": (C.c_int, [C.c_void_p, C.c_int]),
    "fluxmoe_profile_collect": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_uint32)]),
    "fluxmoe_device_errors": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint32)]),
    "fluxmoe_paged_tensor_layout": (C.c_int, [C.POINTER(Desc), C.c_uint64, C.c_uint32,
                                              C.POINTER(PagedTensorInfo)]),
    "fluxmoe_paged_tensor_create": (C.c_int, [C.POINTER(Desc), C.c_void_p, C.POINTER(C.c_void_p)]),
    "fluxmoe_paged_tensor_destroy": (C.c_int, [C.c_void_p]),
    "fluxmoe_paged_tensor_info_get": (C.c_int, [C.c_void_p, C.POINTER(PagedTensorInfo)]),
    "fluxmoe_paged_tensor_address": (C.c_int, [C.c_void_p, C.c_uint32, C.c_int, C.c_uint32,
                                               C.POINTER(C.c_void_p)]),
    "fluxmoe_paged_tensor_set_class": (C.c_int, [C.c_void_p, C.c_uint32, C.c_int]),
    "fluxmoe_balanced_split": (C.c_int, [C.c_double, C.c_double, C.c_uint32, C.POINTER(C.c_double),
                                         C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]),
    "fluxmoe_planner_create": (C.c_int, [C.POINTER(PlannerDesc), C.c_void_p, C.POINTER(C.c_void_p)]),
    "fluxmoe_planner_destroy": (C.c_int, [C.c_void_p]),
    "fluxmoe_planner_max_moves": (C.c_uint32, [C.c_void_p]),
    "fluxmoe_planner_tick": (C.c_int, [C.c_void_p, C.c_uint64, C.c_uint64, C.c_double, C.c_void_p,
                                       C.POINTER(PlannerDecision), C.c_void_p, C.c_size_t]),
    "fluxmoe_planner_reclaim": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.POINTER(C.c_uint32)]),
    "fluxmoe_planner_restore": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.POINTER(C.c_uint32)]),
    "fluxmoe_planner_state": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
}


def lib():
    """Load libfluxmoe.so (once).  Raises if it is missing: there is no other code path."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                _LIB_PATH + " is missing: run `python -m paper_2604_02715_amd.build` "
                "(or __graft_entry__.build()); this package has no non-HIP code path")
        handle = C.CDLL(_LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def _check(rc: int):
    if rc != 0:
        raise FluxmoeError(rc, lib().fluxmoe_last_error().decode())


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def fluxmoe_create(n_layers, n_experts, hidden, ffn, n_slots, block_bytes=4096, max_code_len=12):
    d = Desc(n_layers, n_experts, hidden, ffn, block_bytes, max_code_len, n_slots, 0)
    h = C.c_void_p()
    _check(lib().fluxmoe_create(C.byref(d), C.byref(h)))
    return h


def fluxmoe_destroy(ctx):
    _check(lib().fluxmoe_destroy(ctx))


def fluxmoe_query_sizes(ctx) -> Sizes:
    s = Sizes()
    _check(lib().fluxmoe_query_sizes(ctx, C.byref(s)))
    return s


def fluxmoe_ffn_workspace_bytes(ctx, T, K, shared_expert=False) -> int:
    return int(lib().fluxmoe_ffn_workspace_bytes(ctx, T, K, int(shared_expert)))


def fluxmoe_ffn_plan(ctx, T, K):
    """(rows per tile, K splits of the second product) of the launch plan for T tokens, K experts each."""
    m, k = C.c_uint32(0), C.c_uint32(0)
    _check(lib().fluxmoe_ffn_plan(ctx, T, K, C.byref(m), C.byref(k)))
    return int(m.value), int(k.value)


def fluxmoe_encode_pool(ctx, layer, w13_ptr, w2_ptr, dst_ptr, dst_cap, n_threads=8) -> int:
    used = C.c_size_t(0)
    _check(lib().fluxmoe_encode_pool(ctx, layer, w13_ptr, w2_ptr, dst_ptr, dst_cap, C.byref(used),
                                     n_threads))
    return int(used.value)


def fluxmoe_layer_info_get(ctx, layer) -> LayerInfo:
    info = LayerInfo()
    _check(lib().fluxmoe_layer_info_get(ctx, layer, C.byref(info)))
    return info


def fluxmoe_code_lengths(ctx, layer, type_) -> np.ndarray:
    out = np.zeros(256, dtype=np.uint8)
    _check(lib().fluxmoe_code_lengths(ctx, layer, type_, out.ctypes.data))
    return out


def fluxmoe_tensor_blocks(ctx, layer, type_, expert):
    a, b = C.c_uint64(), C.c_uint64()
    _check(lib().fluxmoe_tensor_blocks(ctx, layer, type_, expert, C.byref(a), C.byref(b)))
    return int(a.value), int(b.value)


def fluxmoe_tensor_first_elems(ctx, layer, type_, expert) -> np.ndarray:
    _, nb = fluxmoe_tensor_blocks(ctx, layer, type_, expert)
    out = np.zeros(nb + 1, dtype=np.uint32)
    _check(lib().fluxmoe_tensor_first_elems(ctx, layer, type_, expert, out.ctypes.data, out.size))
    return out


def fluxmoe_bind_arenas(ctx, slots13_ptr, slots2_ptr, workspace_ptr, workspace_bytes):
    _check(lib().fluxmoe_bind_arenas(ctx, slots13_ptr, slots2_ptr, workspace_ptr, workspace_bytes))


def fluxmoe_bind_layer(ctx, layer, hbm_ptr, n_host_blocks=0, host_ptr=None, check_host_copy_ptr=None):
    _check(lib().fluxmoe_bind_layer(ctx, layer, hbm_ptr, n_host_blocks, host_ptr, check_host_copy_ptr))


def fluxmoe_set_tensor_backing(ctx, layer, type_, expert, tier, blocks_ptr):
    _check(lib().fluxmoe_set_tensor_backing(ctx, layer, type_, expert, tier, blocks_ptr))


def fluxmoe_bind_staging(ctx, staging_ptr, staging_bytes):
    _check(lib().fluxmoe_bind_staging(ctx, staging_ptr, staging_bytes))


def fluxmoe_reset_page_table(ctx, page_table_ptr, stream=None):
    _check(lib().fluxmoe_reset_page_table(ctx, page_table_ptr, stream))


def fluxmoe_prefetch_host(ctx, layer, expert_ids, copy_stream=None):
    ids = _i32(expert_ids)
    _check(lib().fluxmoe_prefetch_host(ctx, layer, ids.ctypes.data, ids.size, copy_stream))


def fluxmoe_materialize(ctx, layer, expert_ids, page_table_ptr, dst_slots, stream=None):
    ids, slots = _i32(expert_ids), _i32(dst_slots)
    if ids.size != slots.size:
        raise ValueError("expert_ids and dst_slots differ in length")
    _check(lib().fluxmoe_materialize(ctx, layer, ids.ctypes.data, ids.size, page_table_ptr,
                                     slots.ctypes.data, stream))


def fluxmoe_materialize_two_streams(ctx, layer, expert_ids, page_table_ptr, dst_slots, stream, stream_type2):
    ids, slots = _i32(expert_ids), _i32(dst_slots)
    if ids.size != slots.size:
        raise ValueError("expert_ids and dst_slots differ in length")
    _check(lib().fluxmoe_materialize_two_streams(ctx, layer, ids.ctypes.data, ids.size, page_table_ptr,
                                                 slots.ctypes.data, stream, stream_type2))


def fluxmoe_release(ctx, layer, expert_ids, page_table_ptr, stream=None):
    if expert_ids is None:
        _check(lib().fluxmoe_release(ctx, layer, None, 0, page_table_ptr, stream))
    else:
        ids = _i32(expert_ids)
        _check(lib().fluxmoe_release(ctx, layer, ids.ctypes.data, ids.size, page_table_ptr, stream))


def fluxmoe_expert_ffn(ctx, layer, tokens_ptr, T, topk_ids_ptr, topk_w_ptr, K, page_table_ptr,
                       out_ptr, flags=0, stream=None):
    _check(lib().fluxmoe_expert_ffn(ctx, layer, tokens_ptr, T, topk_ids_ptr, topk_w_ptr, K,
                                    page_table_ptr, out_ptr, flags, stream))


STATIC_SCRATCH_BYTES = 32 << 20          # FLUXMOE_STATIC_SCRATCH_BYTES


def fluxmoe_expert_ffn_static(ctx, layer, tokens_ptr, T, topk_ids_ptr, topk_w_ptr, K, page_table_ptr,
                              out_ptr, flags=0, stream=None):
    _check(lib().fluxmoe_expert_ffn_static(ctx, layer, tokens_ptr, T, topk_ids_ptr, topk_w_ptr, K,
                                           page_table_ptr, out_ptr, flags, stream))


def fluxmoe_shared_expert_ffn(ctx, w13_ptr, w2_ptr, tokens_ptr, T, out_ptr, flags=0, stream=None):
    _check(lib().fluxmoe_shared_expert_ffn(ctx, w13_ptr, w2_ptr, tokens_ptr, T, out_ptr, flags, stream))


def fluxmoe_stream_copy(dst_ptr, src_ptr, nbytes, n_workgroups, stream=None):
    _check(lib().fluxmoe_stream_copy(dst_ptr, src_ptr, nbytes, n_workgroups, stream))


def fluxmoe_stream_mix(dst_ptr, dst_bytes, src_ptr, src_bytes, out_bytes_small, waves_per_workgroup=8,
                       blocks_per_wave=3, order=0, stream=None):
    """Returns the bytes written."""
    written = C.c_uint64(0)
    _check(lib().fluxmoe_stream_mix(dst_ptr, dst_bytes, src_ptr, src_bytes, out_bytes_small, waves_per_workgroup,
                                    blocks_per_wave, order, C.byref(written), stream))
    return int(written.value)


def fluxmoe_mfma_probe(operands_ptr, out_ptr, n_workgroups, iters, stream=None):
    _check(lib().fluxmoe_mfma_probe(operands_ptr, out_ptr, n_workgroups, iters, stream))


PROFILE_KINDS = ("decode", "grouping", "gemm1_swiglu", "gemm2", "combine")


def fluxmoe_profile_enable(ctx, on: bool, only_kinds=None):
    """only_kinds: names from PROFILE_KINDS; None = every kind."""
    v = int(bool(on))
    if on and only_kinds is not None:
        v = 0x100 | sum(1 << PROFILE_KINDS.index(k) for k in only_kinds)
    _check(lib().fluxmoe_profile_enable(ctx, v))


def fluxmoe_profile_collect(ctx) -> dict:
    """{kind: (total_ms, launches)} since the last collect."""
    ms = (C.c_double * 5)()
    cnt = (C.c_uint32 * 5)()
    _check(lib().fluxmoe_profile_collect(ctx, ms, cnt))
    return {k: (float(ms[i]), int(cnt[i])) for i, k in enumerate(PROFILE_KINDS)}


def fluxmoe_device_errors(ctx) -> int:
    f = C.c_uint32(0)
    _check(lib().fluxmoe_device_errors(ctx, C.byref(f)))
    return int(f.value)


# ---------------------------------------------------------------------- residency planner
def fluxmoe_planner_create(n_layers, experts_per_rank, control_interval=0, theta=0.0,
                           adjustment_granularity=0.0, uncompressed=None):
    d = PlannerDesc(n_layers, experts_per_rank, control_interval, 0, theta, adjustment_granularity)
    h = C.c_void_p()
    flags = None
    if uncompressed is not None:
        flags = np.ascontiguousarray(uncompressed, dtype=np.uint8)
        if flags.size != n_layers:
            raise ValueError("uncompressed must have n_layers entries")
    _check(lib().fluxmoe_planner_create(C.byref(d), None if flags is None else flags.ctypes.data,
                                        C.byref(h)))
    return h


def fluxmoe_planner_destroy(p):
    _check(lib().fluxmoe_planner_destroy(p))


def fluxmoe_planner_max_moves(p) -> int:
    return int(lib().fluxmoe_planner_max_moves(p))


def _moves_list(buf, n):
    return [(int(m.layer), int(m.expert), int(m.type), int(m.to_host)) for m in buf[:n]]


def fluxmoe_planner_tick(p, B_rem, B_act, tau_fwd, tau_load_layer=None):
    """(decision, [(layer, expert, type, to_host), ...])"""
    cap = fluxmoe_planner_max_moves(p)
    buf = (PlannerMove * cap)()
    dec = PlannerDecision()
    loads = None if tau_load_layer is None else np.ascontiguousarray(tau_load_layer, dtype=np.float64)
    _check(lib().fluxmoe_planner_tick(p, B_rem, B_act, tau_fwd,
                                      None if loads is None else loads.ctypes.data, C.byref(dec),
                                      C.cast(buf, C.c_void_p), cap))
    return dec, _moves_list(buf, dec.n_moves)


def _planner_step(fn, p):
    cap = fluxmoe_planner_max_moves(p)
    buf = (PlannerMove * cap)()
    n = C.c_uint32(0)
    _check(fn(p, C.cast(buf, C.c_void_p), cap, C.byref(n)))
    return _moves_list(buf, n.value)


def fluxmoe_planner_reclaim(p):
    return _planner_step(lib().fluxmoe_planner_reclaim, p)


def fluxmoe_planner_restore(p):
    return _planner_step(lib().fluxmoe_planner_restore, p)


def fluxmoe_planner_state(p, n_layers, experts_per_rank):
    """(layer_pageable uint8 [N], on_host uint8 [N][L_r][2]; last index 0 = type 1, 1 = type 2)"""
    pageable = np.zeros(n_layers, dtype=np.uint8)
    on_host = np.zeros((n_layers, experts_per_rank, 2), dtype=np.uint8)
    _check(lib().fluxmoe_planner_state(p, pageable.ctypes.data, on_host.ctypes.data))
    return pageable, on_host


def fluxmoe_balanced_split(beta_gpu, beta_cpu, experts_per_rank):
    """(x_bw, n_down, n_fused)"""
    x, nd, nf = C.c_double(), C.c_uint32(), C.c_uint32()
    _check(lib().fluxmoe_balanced_split(beta_gpu, beta_cpu, experts_per_rank, C.byref(x), C.byref(nd),
                                        C.byref(nf)))
    return float(x.value), int(nd.value), int(nf.value)


# ---------------------------------------------------------------------- PagedTensor (VMM)
def _desc(n_layers, n_experts, hidden, ffn):
    return Desc(n_layers, n_experts, hidden, ffn, 4096, 12, 2 * n_experts, 0)


def fluxmoe_paged_tensor_layout(n_layers, n_experts, hidden, ffn, granularity, n_uncompressed=0):
    d, info = _desc(n_layers, n_experts, hidden, ffn), PagedTensorInfo()
    _check(lib().fluxmoe_paged_tensor_layout(C.byref(d), granularity, n_uncompressed, C.byref(info)))
    return info


def fluxmoe_paged_tensor_create(n_layers, n_experts, hidden, ffn, uncompressed=None):
    d, h = _desc(n_layers, n_experts, hidden, ffn), C.c_void_p()
    flags = None
    if uncompressed is not None:
        flags = np.ascontiguousarray(uncompressed, dtype=np.uint8)
        if flags.size != n_layers:
            raise ValueError("uncompressed must have n_layers entries")
    _check(lib().fluxmoe_paged_tensor_create(C.byref(d), None if flags is None else flags.ctypes.data,
                                             C.byref(h)))
    return h


def fluxmoe_paged_tensor_destroy(p):
    _check(lib().fluxmoe_paged_tensor_destroy(p))


def fluxmoe_paged_tensor_info_get(p) -> PagedTensorInfo:
    info = PagedTensorInfo()
    _check(lib().fluxmoe_paged_tensor_info_get(p, C.byref(info)))
    return info


def fluxmoe_paged_tensor_address(p, layer, type_, expert) -> int:
    out = C.c_void_p()
    _check(lib().fluxmoe_paged_tensor_address(p, layer, type_, expert, C.byref(out)))
    return int(out.value)


def fluxmoe_paged_tensor_set_class(p, layer, uncompressed: bool):
    _check(lib().fluxmoe_paged_tensor_set_class(p, layer, int(uncompressed)))
