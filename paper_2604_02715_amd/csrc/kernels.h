// Device-side structures and kernel launchers of libfluxmoe.so (decode side: decode_args.h).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "decode_args.h"

namespace fluxmoe {

// ---------------------------------------------------------------- expert FFN
struct FfnArgs {
    const uint16_t* tokens;      // BF16 [T][H]
    const int32_t* topk_ids;     // [T][K]
    const float* topk_w;         // [T][K]
    const int32_t* page_table;   // this layer's row: [n_experts]
    const uint16_t* slots13;     // type-1 arena
    const uint16_t* slots2;      // type-2 arena
    float* out;                  // [T][H]
    uint32_t T, K, H, F, E;
    uint32_t flags;
    // workspace carve-up (device)
    int32_t* expert_count;       // [E + 1]
    int32_t* expert_offset;      // [E + 2]
    int32_t* sorted_pair;        // [pairs_cap]  pair index (t * K + k), grouped by expert
    int32_t* pair_pos;           // [pairs_cap]  position of a pair in sorted order, -1 = skipped
    int4* tile_rec;              // [tiles_cap]  (expert, first sorted row, rows, slot); rows = 0 past the last tile
    int32_t* n_tiles;            // [1]
    int32_t* chunk_count;        // [n_chunks][E]  large batches: pairs per (chunk of kRouteChunkPairs pairs, expert),
                                 // turned into the chunk's first position inside the expert's rows by the grouping kernel
    uint32_t n_chunks;           // 0: the grouping kernel counts and scatters the pairs itself (one workgroup)
    uint16_t* hbuf;              // BF16 [pairs_cap][F]
    float* ybuf;                 // FP32 [ksplit][pairs_cap][H]
    uint32_t* error_word;
    uint32_t pairs_cap, tiles_cap, m_tile, ksplit;
    uint32_t tiled_waves;        // variant of the LDS-tiled kernels (m_tile 256): 2 LDS-direct loads, 8 or 4
                                 // wavefronts with register-staged loads
    uint32_t tiled_persist;      // LDS-direct kernels: workgroups per CU-sized round that walk through the tiles (1 = 256
                                 // workgroups), 0 = one workgroup per tile
    uint32_t tiled_sn_log2;      // set per launch by launch_ffn: log2 of the columns of the LDS-direct kernels' super-tile
    uint32_t tiled_total;        // set per launch by launch_ffn: tile numbers of the LDS-direct kernel's launch
    uint32_t tiled_group;        // super-rows of the LDS-direct gate/up kernel that share a column block in time;
                                 // 0 = launch_ffn derives it from the rows per expert
};

// Batches with more pairs than this are counted and scattered by one workgroup per kRouteChunkPairs pairs
// around the single workgroup that scans the experts (a single workgroup needs 0.4 ms for 330000 pairs).
constexpr uint32_t kRouteChunkThreshold = 32768;
constexpr uint32_t kRouteChunkPairs = 8192;

// hook(user, kind, begin, stream) is called around every kernel when timing is on
// (kinds: 1 grouping, 2 gate/up product + SwiGLU, 3 down product, 4 combine)
typedef void (*SpanHook)(void* user, int kind, int begin, hipStream_t stream);
hipError_t launch_ffn(const FfnArgs& args, int n_cus, hipStream_t stream, SpanHook hook, void* user);
hipError_t launch_mfma_probe(const void* operands, float* out, uint32_t n_workgroups, uint32_t iters,
                             hipStream_t stream);
// The decode kernel's launch shape and memory accesses without its work (probe_kernels.hip): n_blocks blocks of
// 4096 bytes read, stream_mix_out_bytes(n_blocks, small) bytes written (small or small + 128 bytes per block).
uint64_t stream_mix_out_bytes(uint64_t n_blocks, uint32_t small);
hipError_t launch_stream_mix(void* dst, const void* src, uint32_t n_blocks, uint32_t small, int waves_per_wg,
                             uint32_t per_wave, uint32_t order, uint32_t n_workgroups, hipStream_t stream);

}  // namespace fluxmoe
